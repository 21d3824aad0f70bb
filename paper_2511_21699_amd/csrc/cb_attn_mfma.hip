// Tree-masked flash-decode attention on the matrix cores (bf16, head_dim 128), gfx950 only.
//
// Tree attention, Section 3.2 of the paper: node i attends to the KV-cached prefix (slots 0..S-1)
// and to the tree nodes on its own ancestor chain (slots S+a, a in anc(i)).  For one kv head the
// g*N query rows (g query heads per kv head, N nodes) form a small dense matrix, so QK^T and PV are
// MFMA contractions; the KV sequence is split across workgroups and the partial softmax states
// (o, m, l) are merged afterwards.
//
// Work decomposition: one workgroup (4 or 8 wavefronts, see attn_tile) per (sequence, kv head, row
// tile, split).  A wave owns 16*R rows; K/V stages are brought straight from HBM into an LDS
// ring by LDS-DMA (global_load_lds: no registers held by loads in flight) and are shared by the
// waves.  All loads of the sweep -- the ring's requests, the query rows, a logits item -- are issued
// as instructions the compiler does not interpret and are covered by the kernel's own counted waits
// (lds_dma_b128, load_b128_untracked).
//
// Register layouts (v_mfma_f32_16x16x32_bf16; lane l, c = l%16, kg = l/16):
//   scores are computed transposed, S^T = K Q^T: A = K rows (key c of the sub-tile, dims
//   8kg..8kg+7 of the 32-dim step), B = Q^T (query c, same dims), D[v] = S^T[key 4kg+v][query c].
//   A lane therefore holds 4 keys x 1 query per 16-key sub-tile: softmax statistics are per-lane
//   scalars shared by the 4 lanes with equal c.
//   O^T = V^T P^T: B = P^T packs the lane's 8 probabilities of a 32-key tile (element e <-> key
//   16(e/4)+4kg+e%4), A = V^T must hold the same keys for dim c of the 16-dim tile; it is fetched
//   from the row-major V tile with ds_read_b64_tr_b16 (each 16-lane group reads a 4-key x 16-dim
//   block and receives it transposed).  D[v] = O^T[dim 4kg+v][query c].
#include <type_traits>

#include "cb_logits.h"

namespace cb {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(4 * sizeof(unsigned)))) unsigned uintx4;
typedef __attribute__((__vector_size__(2 * sizeof(unsigned)))) unsigned uintx2;
#define CB_GLOBAL __attribute__((address_space(1)))
#define CB_LDS __attribute__((address_space(3)))
constexpr int kAgentCoherent = 16;  // buffer cache policy: sc1 = coherent at agent (device) scope

constexpr int kStageKeys = 32;                 // keys per half-stage: the unit of the LDS ring, one wave group's share of a stage
constexpr int kStageVecs = kStageKeys * 16;    // 16-byte pieces per K (or V) half-stage: 32 rows x 256 B
constexpr int NH = 9;                          // ring depth in half-stages (16 KiB each): 288 keys
constexpr int PRO = 6;                         // half-stages requested before the first wait; the rest of the ring right after it
constexpr int kMaxBtLds = 1024;                // block-table entries staged in LDS per split
// Partial softmax state in this kernel's own format, one unit per (16-row tile, split), laid out in
// the order the MFMA accumulators hold it: for each of the 8 dim tiles dt, lane (kg, c) of the wave
// that owns the 16 rows has 8 bytes -- o[row c][16 dt + 4 kg + {0..3}] as bf16, unnormalised, relative
// to the reference weight -- at dt * 512 + lane * 8, so that a wave's store or load of one dim tile is
// 512 contiguous bytes; then (m, l) as fp32 for each of the 16 rows.  bf16 halves the bytes, which
// matters because one workgroup pulls all partials of its tile through a single compute unit.
// The units of sequence b start at tile unit_tile0(b); kv head hk's row tile ti (16 rows) is unit
// (hk * ceil(M_b / 16) + ti) * nsplit + split behind it.
constexpr int kUnitMl = 8 * 512;
constexpr int kUnitBytes = kUnitMl + 16 * 8;
// first 16-row tile of a sequence whose nodes start at `off`: room for ceil(M_b / 16) tiles per kv
// head without a prefix sum over the sequences' tile counts
__host__ __device__ __forceinline__ int64_t unit_tile0(int64_t off, int Hq, int Hkv, int b) {
  return ((off * Hq) >> 4) + (int64_t)(Hkv + 1) * b;
}


template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt simm16 on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// A 16-byte global load that the compiler does not know to be one.  It orders every load it tracks
// against the LDS-DMA requests of the ring as if the two kinds could overtake each other: the first
// use of a tracked load's result while ring requests are in flight costs a wait for all of them.
// Loads return in the order they were issued, so the ring's own counted waits cover these; the
// caller pins the result (asm "+v") behind such a wait before it touches it.
__device__ __forceinline__ uintx4 load_b128_untracked(const CB_GLOBAL void* p) {
  uintx4 r;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}

__device__ __forceinline__ uint16_t f2bf(float x) {
  uint32_t u = __float_as_uint(x);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct KeyAddr {  // resolves cache slots of one (sequence, kv head) to byte offsets
  const KvAddr* kv;
  const int* bt;   // LDS copy of this split's slice of the block table (paged caches)
  int bt_first;    // logical block of bt[0]
  int bs_shift;    // log2(block_size)
  int seq, head;
  __device__ __forceinline__ int64_t byte_off(int slot) const {
    const KvAddr& a = *kv;
    if (a.block_size > 0) {
      const int lb = slot >> bs_shift;
      int64_t blk = bt[lb - bt_first];
      blk = blk < 0 ? 0 : (blk >= a.num_blocks ? a.num_blocks - 1 : blk);
      return (blk * a.seq_stride + (int64_t)(slot - (lb << bs_shift)) * a.token_stride +
              (int64_t)head * a.head_stride) * 2;
    }
    return ((int64_t)seq * a.seq_stride + (int64_t)slot * a.token_stride + (int64_t)head * a.head_stride) * 2;
  }
};

// Workgroup barrier without the memory fence of __syncthreads(): the fence would wait for every
// outstanding global->LDS load (vmcnt 0) and serialise the ring.  Ordering of LDS traffic is by
// construction: a wave waits for its own loads of the stage (s_waitcnt vmcnt) before the barrier,
// and every LDS read of the previous stage has been consumed by an MFMA before it.  The empty asm
// statements stop the compiler from moving memory accesses across.
__device__ __forceinline__ void ring_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// One LDS-DMA request: every lane's 16 bytes at `src` go to LDS at dst + lane * 16 (dst is the same
// in all lanes of the wave).  Written as an instruction the compiler does not interpret: for the
// builtin it keeps its own account of which request has landed, cannot relate the ring's counted
// waits to the conditional refills, and puts a wait for everything in flight in front of the
// stages' LDS reads (and in front of the loop, for the query registers).  Here every wait is the
// ring's own: a stage's wait and barrier come before any read of its slot, and each of these
// statements is a compiler barrier for memory accesses.
__device__ __forceinline__ void lds_dma_b128(const CB_GLOBAL char* src, CB_LDS uint4* dst) {
  const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory");
}

// Wave `w` (of 8) brings rows 4w..4w+3 of a half-stage (keys key0..key0+31) into its ring slot: one
// 1 KiB request for K and one for V.  LDS position of a 16-byte piece is fixed by the lane
// (row*16 + c); which piece of the row lands there is chosen by the XOR swizzle so that the MFMA
// operand reads below are free of bank conflicts.  Keys past `last_key` repeat it (they are never
// used), so every address stays inside the split's own range.
__device__ __forceinline__ void issue_half(uint4* kdst, uint4* vdst, const KeyAddr& ka, const CB_GLOBAL char* kbase,
                                           const CB_GLOBAL char* vbase, int key0, int last_key, int w, int l) {
  const int r = 4 * w + (l >> 4);
  const int c = l & 15;
  int key = key0 + r;
  key = key > last_key ? last_key : key;
  const int64_t off = ka.byte_off(key);
  const int pk = c ^ (r & 15);
  const int pv = c ^ ((r & 7) << 1);
  lds_dma_b128(kbase + off + pk * 16, (CB_LDS uint4*)kdst + (4 * w) * 16);
  lds_dma_b128(vbase + off + pv * 16, (CB_LDS uint4*)vdst + (4 * w) * 16);
}

template <int R>
struct WaveState {
  bf16x8 q[R][4];    // B operands of QK^T: query c, dims 32*ds + 8kg ..
  floatx4 o[R][8];   // O^T accumulators, 8 dim tiles of 16
  floatx4 lacc[R];   // softmax denominator, accumulated by an MFMA against a tile of ones
  float mref[R];     // reference maximum of the raw scores (q.k, before the softmax scale)
};

// Maximum over the 4 lanes that share a query (lanes c, c+16, c+32, c+48) with the gfx950 row
// swaps: v_permlane16_swap exchanges odd 16-lane rows of one operand with even rows of the other,
// v_permlane32_swap the upper half of one with the lower half of the other, so two swaps of a
// value with itself bring every lane its partners.
// max of two finite-or-infinite floats as a median with +inf: one v_med3_f32, where fmaxf() costs a
// canonicalising v_max_f32 per operand first (the compiler cannot know that MFMA results are not
// signalling NaNs; the inputs are finite by precondition, so they are not).
// `pinf` is +inf in a register the compiler cannot see through (opaque_inf()): with a literal it
// folds the median back into fmaxf.
__device__ __forceinline__ float opaque_inf() {
  float x = INFINITY;
  asm("" : "+v"(x));
  return x;
}
__device__ __forceinline__ float max2(float a, float b, float pinf) { return __builtin_amdgcn_fmed3f(a, b, pinf); }
__device__ __forceinline__ float quad_max(float x, float pinf) {
  auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = max2(__uint_as_float(a[0]), __uint_as_float(a[1]), pinf);
  auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return max2(__uint_as_float(b[0]), __uint_as_float(b[1]), pinf);
}

constexpr float kRescaleSlack = 8.0f;  // log2 units the running maximum may exceed the reference

// One 32-key stage for the 16*R rows of a wave.
//   scores  S^T = K Q^T                       (8 MFMAs per row tile)
//   p = 2^(c*s - c*mref) with c = scale*log2(e); mref follows the running maximum lazily: it is
//   only raised (and O, l rescaled) when the maximum has grown by more than kRescaleSlack, so
//   probabilities stay below 2^8 and the accumulators are rarely touched by the vector ALU
//   O^T += V^T P^T, l += 1^T P^T              (9 MFMAs per row tile)
// NV <= R is the number of leading row tiles of the wave that hold real rows; the others are skipped.
template <int R, int NV>
__device__ __forceinline__ void compute_stage(const uint4* __restrict__ ks, const uint4* __restrict__ vs,
                                              WaveState<R>& st, float c2, int key0, int S, int kend,
                                              bool need_mask, const uint32_t* anc_lds, const int* row_node, int l) {
  const int c = l & 15, kg = l >> 4;
  const float pinf = opaque_inf();
  // all K operands of the stage are requested before the first MFMA, and all V operands before the
  // softmax arithmetic, so that LDS latency hides behind the matrix and vector work
  uint4 kraw[2][4];
#pragma unroll
  for (int sub = 0; sub < 2; sub++) {
    const int row = 16 * sub + c;
#pragma unroll
    for (int ds = 0; ds < 4; ds++) kraw[sub][ds] = ks[row * 16 + ((kg + 4 * ds) ^ (row & 15))];
  }
  // (with one row tile per wave the V operands are also requested up front; with two, the MFMA work
  // per LDS byte is twice as large and the registers are needed for the accumulators instead)
  const char* vbytes = reinterpret_cast<const char*>(vs);
  constexpr int kHoistV = R == 1 ? 8 : 4;  // dim tiles whose V operands are read before the softmax
  bf16x4 va[8][2];
  auto read_v = [&](int dt) {
#pragma unroll
    for (int t = 0; t < 2; t++) {
      const int row = 16 * t + 4 * kg + (c >> 2);
      const int piece = 2 * dt + ((c & 3) >> 1);
      const int slot = piece ^ ((row & 7) << 1);
      const char* addr = vbytes + row * 256 + slot * 16 + (c & 1) * 8;
      va[dt][t] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(addr));
    }
  };
#pragma unroll
  for (int dt = 0; dt < kHoistV; dt++) read_v(dt);
  floatx4 s[NV][2];
#pragma unroll
  for (int rr = 0; rr < NV; rr++) {
    s[rr][0] = floatx4{0.f, 0.f, 0.f, 0.f};
    s[rr][1] = floatx4{0.f, 0.f, 0.f, 0.f};
  }
#pragma unroll
  for (int ds = 0; ds < 4; ds++) {
#pragma unroll
    for (int sub = 0; sub < 2; sub++) {
      const bf16x8 a = __builtin_bit_cast(bf16x8, kraw[sub][ds]);
#pragma unroll
      for (int rr = 0; rr < NV; rr++)
        s[rr][sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, st.q[rr][ds], s[rr][sub], 0, 0, 0);
    }
  }
  bf16x8 pb[NV];
#pragma unroll
  for (int rr = 0; rr < NV; rr++) {
    float x[8];
#pragma unroll
    for (int e = 0; e < 8; e++) x[e] = s[rr][e >> 2][e & 3];
    if (need_mask) {
      // 32-bit visibility word of this stage for the lane's query: bit j <-> key key0 + j.
      const uint32_t* arow = anc_lds + row_node[rr] * kAncWords;
      const int np = S - key0;     // prefix keys in the stage (may be <= 0 or >= 32)
      const int ne = kend - key0;  // keys before the split's end (>= 1)
      uint32_t vis = np >= 32 ? 0xffffffffu : (np <= 0 ? 0u : ((1u << np) - 1u));
      if (np < 32) {
        uint32_t tree;
        if (np > 0) {
          tree = arow[0] << np;  // tree node 0 sits at bit np
        } else {
          const int t0 = -np, w0 = t0 >> 5, sh = t0 & 31;
          const uint32_t lo = w0 < kAncWords ? arow[w0] : 0u;
          const uint32_t hi = (w0 + 1 < kAncWords) ? arow[w0 + 1] : 0u;
          tree = sh ? ((lo >> sh) | (hi << (32 - sh))) : lo;
        }
        vis |= tree;
      }
      if (ne < 32) vis &= (1u << ne) - 1u;  // keys past the split's end belong to the next split (or do not exist)
#pragma unroll
      for (int e = 0; e < 8; e++) {
        const int j = 16 * (e >> 2) + 4 * kg + (e & 3);
        x[e] = ((vis >> j) & 1u) ? x[e] : -INFINITY;
      }
    }
    float mx = max2(max2(max2(x[0], x[1], pinf), max2(x[2], x[3], pinf), pinf),
                    max2(max2(x[4], x[5], pinf), max2(x[6], x[7], pinf), pinf), pinf);
    mx = quad_max(mx, pinf);
    // lazy reference update; the decision is identical in the 4 lanes of a query
    const bool raise = (mx - st.mref[rr]) * c2 > kRescaleSlack;  // false when both are -inf (NaN)
    if (__builtin_amdgcn_ballot_w64(raise) != 0ull) {
      const float alpha = raise ? __builtin_amdgcn_exp2f((st.mref[rr] - mx) * c2) : 1.0f;
      if (raise) st.mref[rr] = mx;
#pragma unroll
      for (int dt = 0; dt < 8; dt++) st.o[rr][dt] *= alpha;
      st.lacc[rr] *= alpha;
    }
    const float nm = (st.mref[rr] == -INFINITY) ? 0.f : -st.mref[rr] * c2;
    union { bf16x8 v; __bf16 h[8]; } pk;
#pragma unroll
    for (int e = 0; e < 8; e++) pk.h[e] = (__bf16)__builtin_amdgcn_exp2f(fmaf(x[e], c2, nm));
    pb[rr] = pk.v;
  }
  // O^T += V^T P^T and l += 1^T P^T
  const bf16x8 ones = __builtin_bit_cast(bf16x8, uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
#pragma unroll
  for (int rr = 0; rr < NV; rr++)
    st.lacc[rr] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[rr], st.lacc[rr], 0, 0, 0);
#pragma unroll
  for (int dt = 0; dt < 8; dt++) {
    if (dt + 4 < 8 && dt + 4 >= kHoistV) read_v(dt + 4);  // keep four dim tiles of V ahead of the MFMAs
    const bf16x8 a = __builtin_shufflevector(va[dt][0], va[dt][1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
    for (int rr = 0; rr < NV; rr++)
      st.o[rr][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, pb[rr], st.o[rr][dt], 0, 0, 0);
  }
}

// The same stage for a wave with two full row tiles and no key to mask (all keys in the cached
// prefix and inside the split): the common case of long sweeps.  The two row tiles are independent
// chains QK^T -> softmax -> PV; written one behind the other they leave the matrix cores idle during
// the softmax and the vector ALU idle during the MFMAs.  Here the second tile's exponentials are
// spread between the first tile's PV MFMAs (an MFMA occupies the matrix core for 16 cycles during
// which the wave can issue independent vector instructions), and the row maxima of both tiles are
// taken before a single, rarely taken rescale branch, so that everything after it is one basic block.
__device__ __forceinline__ void compute_stage_pair(const uint4* __restrict__ ks, const uint4* __restrict__ vs,
                                                   WaveState<2>& st, float c2, int l) {
  const int c = l & 15, kg = l >> 4;
  const float pinf = opaque_inf();
  uint4 kraw[2][4];
#pragma unroll
  for (int sub = 0; sub < 2; sub++) {
    const int row = 16 * sub + c;
#pragma unroll
    for (int ds = 0; ds < 4; ds++) kraw[sub][ds] = ks[row * 16 + ((kg + 4 * ds) ^ (row & 15))];
  }
  const char* vbytes = reinterpret_cast<const char*>(vs);
  bf16x4 va[8][2];
  auto read_v = [&](int dt) {
#pragma unroll
    for (int t = 0; t < 2; t++) {
      const int row = 16 * t + 4 * kg + (c >> 2);
      const int piece = 2 * dt + ((c & 3) >> 1);
      const int slot = piece ^ ((row & 7) << 1);
      const char* addr = vbytes + row * 256 + slot * 16 + (c & 1) * 8;
      va[dt][t] = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((bf16x4 __attribute__((address_space(3)))*)(addr));
    }
  };
#pragma unroll
  for (int dt = 0; dt < 4; dt++) read_v(dt);
  // ---- scores of both tiles, tile 0 first so that its maximum can be taken under tile 1's MFMAs
  floatx4 s[2][2];
  float mx[2];
#pragma unroll
  for (int rr = 0; rr < 2; rr++) {
    s[rr][0] = floatx4{0.f, 0.f, 0.f, 0.f};
    s[rr][1] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ds = 0; ds < 4; ds++) {
#pragma unroll
      for (int sub = 0; sub < 2; sub++)
        s[rr][sub] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kraw[sub][ds]), st.q[rr][ds], s[rr][sub], 0, 0, 0);
    }
  }
  bool raise[2];
#pragma unroll
  for (int rr = 0; rr < 2; rr++) {
    float m = max2(max2(max2(s[rr][0][0], s[rr][0][1], pinf), max2(s[rr][0][2], s[rr][0][3], pinf), pinf),
                   max2(max2(s[rr][1][0], s[rr][1][1], pinf), max2(s[rr][1][2], s[rr][1][3], pinf), pinf), pinf);
    mx[rr] = quad_max(m, pinf);
    raise[rr] = (mx[rr] - st.mref[rr]) * c2 > kRescaleSlack;  // false when both are -inf (NaN)
  }
  if (__builtin_amdgcn_ballot_w64(raise[0] || raise[1]) != 0ull) {
#pragma unroll
    for (int rr = 0; rr < 2; rr++) {
      const float alpha = raise[rr] ? __builtin_amdgcn_exp2f((st.mref[rr] - mx[rr]) * c2) : 1.0f;
      if (raise[rr]) st.mref[rr] = mx[rr];
#pragma unroll
      for (int dt = 0; dt < 8; dt++) st.o[rr][dt] *= alpha;
      st.lacc[rr] *= alpha;
    }
  }
  // ---- one basic block from here on
  const bf16x8 ones = __builtin_bit_cast(bf16x8, uint4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});
  const float nm0 = (st.mref[0] == -INFINITY) ? 0.f : -st.mref[0] * c2;
  const float nm1 = (st.mref[1] == -INFINITY) ? 0.f : -st.mref[1] * c2;
  union { bf16x8 v; __bf16 h[8]; } p0, p1;
#pragma unroll
  for (int e = 0; e < 8; e++) p0.h[e] = (__bf16)__builtin_amdgcn_exp2f(fmaf(s[0][e >> 2][e & 3], c2, nm0));
  // (the scheduling barriers pin this interleaving: left alone, the instruction scheduler gathers all
  // exponentials in front of the MFMAs)
  __builtin_amdgcn_sched_barrier(0);
  st.lacc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, p0.v, st.lacc[0], 0, 0, 0);
  float e1[8];
#pragma unroll
  for (int dt = 0; dt < 8; dt++) {
    if (dt + 4 < 8) read_v(dt + 4);
    const bf16x8 a = __builtin_shufflevector(va[dt][0], va[dt][1], 0, 1, 2, 3, 4, 5, 6, 7);
    st.o[0][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, p0.v, st.o[0][dt], 0, 0, 0);
    e1[dt] = __builtin_amdgcn_exp2f(fmaf(s[1][dt >> 2][dt & 3], c2, nm1));  // tile 1's softmax under tile 0's MFMAs
    asm volatile("" : "+v"(e1[dt]));  // (the value is produced here, not sunk to its use after the loop)
    __builtin_amdgcn_sched_barrier(0);
  }
#pragma unroll
  for (int e = 0; e < 8; e++) p1.h[e] = (__bf16)e1[e];
  st.lacc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, p1.v, st.lacc[1], 0, 0, 0);
#pragma unroll
  for (int dt = 0; dt < 8; dt++) {
    const bf16x8 a = __builtin_shufflevector(va[dt][0], va[dt][1], 0, 1, 2, 3, 4, 5, 6, 7);
    st.o[1][dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, p1.v, st.o[1][dt], 0, 0, 0);
  }
}

// Forces every field of the argument block into scalar registers here and now: the empty asm
// statements take each value as an in/out operand, so the loads cannot be sunk past this point.
#define CB_PIN(x) asm volatile("" : "+s"(x))
__device__ __forceinline__ void pin_args(AttnParams& p) {
  CB_PIN(p.q); CB_PIN(p.out); CB_PIN(p.kv.k); CB_PIN(p.kv.v); CB_PIN(p.kv.block_table);
  CB_PIN(p.kv.seq_stride); CB_PIN(p.kv.token_stride); CB_PIN(p.kv.head_stride); CB_PIN(p.kv.num_blocks);
  CB_PIN(p.kv.max_blocks); CB_PIN(p.kv.block_size); CB_PIN(p.parent); CB_PIN(p.partial); CB_PIN(p.tickets); CB_PIN(p.coop_tickets);
  CB_PIN(p.Hq); CB_PIN(p.Hkv); CB_PIN(p.chunk); CB_PIN(p.nsplit); CB_PIN(p.batch); CB_PIN(p.scale);
  CB_PIN(p.external_merge); CB_PIN(p.max_depth); CB_PIN(p.xcd_remap); CB_PIN(p.grid_x); CB_PIN(p.grid_y); CB_PIN(p.grid_z); CB_PIN(p.coop_merge); CB_PIN(p.spin_limit);
  CB_PIN(p.status); CB_PIN(p.dbg_ts);
}
__device__ __forceinline__ void pin_logits_args(LogitsWork& w) {
  // (what the item's scan needs; the acceptance's own arguments are fetched by the one workgroup
  // that runs it, when it does)
  CB_PIN(w.logits); CB_PIN(w.V); CB_PIN(w.rows); CB_PIN(w.batch); CB_PIN(w.partial_out);
  CB_PIN(w.tickets); CB_PIN(w.accept.slot_stride); CB_PIN(w.accept.nchunks);
}
#undef CB_PIN

// Split merge of one tile by the waves that swept it: every lane merges the elements it held --
// its query row, dims 16 dt + 4 kg + {0..3} of NDT dim tiles from dt0 -- which is also how the
// partials are laid out, so each load of a wave is 512 contiguous bytes (ubyte[rr]: byte offset of
// slot 0's unit of the lane's rr-th row tile).  Slots are combined online, BS per batch with all
// of a batch's loads in flight together: m = max m_t, w_t = 2^(m_t - m),
// o = sum w_t o_t / sum w_t l_t (m_t is stored in log2 units).  POL is the buffer cache policy of
// the loads.  A slot that saw no visible key carries m_t = -inf, l_t = 0 and gets weight 0; the
// reference is kept finite so that (-inf) - (-inf) never occurs.
template <int R, int NDT, int POL, int BS = 32 / NDT>
__device__ __forceinline__ void merge_tile(__amdgpu_buffer_rsrc_t prsrc, const int64_t* grow, const uint32_t* ubyte,
                                           CB_GLOBAL uint16_t* gout, int nslots, int dt0, int l) {
  constexpr int D = 128;
  const int kg = l >> 4, c = l & 15;
#pragma unroll
  for (int rr = 0; rr < R; rr++) {
    if (grow[rr] < 0) continue;
    floatx4 acc[NDT];
#pragma unroll
    for (int i = 0; i < NDT; i++) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
    float lsum = 0.f, m_run = -3.0e38f;
    // (the slot's offset is the same in all lanes: it travels as the load's scalar offset, so a
    // load costs no vector arithmetic)
    const uint32_t vo_ml = ubyte[rr] + kUnitMl + c * 8, vo_v = ubyte[rr] + dt0 * 512 + l * 8;
    for (int t0 = 0; t0 < nslots; t0 += BS) {
      uintx2 v[BS][NDT];
      uintx2 ml[BS];
#pragma unroll
      for (int u = 0; u < BS; u++) {
        const int t = (t0 + u < nslots) ? t0 + u : nslots - 1;  // (a repeated slot: weight 0 below)
        ml[u] = __builtin_amdgcn_raw_buffer_load_b64(prsrc, vo_ml, t * kUnitBytes, POL);
#pragma unroll
        for (int i = 0; i < NDT; i++)
          v[u][i] = __builtin_amdgcn_raw_buffer_load_b64(prsrc, vo_v + i * 512, t * kUnitBytes, POL);
      }
      // (all of the batch's loads are requested before anything looks at a result: left alone, the
      // scheduler moves the first maxima up between the loads, and each then waits a round trip)
      __builtin_amdgcn_sched_barrier(0);
      float m_new = m_run;
#pragma unroll
      for (int u = 0; u < BS; u++) m_new = fmaxf(m_new, __uint_as_float(ml[u][0]));
      if (t0 > 0) {  // (uniform)
        const float resc = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
        for (int i = 0; i < NDT; i++) acc[i] *= resc;
        lsum *= resc;
      }
      m_run = m_new;
#pragma unroll
      for (int u = 0; u < BS; u++) {
        float wgt = __builtin_amdgcn_exp2f(__uint_as_float(ml[u][0]) - m_new);
        wgt = (t0 + u < nslots) ? wgt : 0.f;
        lsum = fmaf(__uint_as_float(ml[u][1]), wgt, lsum);
#pragma unroll
        for (int i = 0; i < NDT; i++) {
          acc[i][0] = fmaf(__uint_as_float(v[u][i][0] << 16), wgt, acc[i][0]);
          acc[i][1] = fmaf(__uint_as_float(v[u][i][0] & 0xffff0000u), wgt, acc[i][1]);
          acc[i][2] = fmaf(__uint_as_float(v[u][i][1] << 16), wgt, acc[i][2]);
          acc[i][3] = fmaf(__uint_as_float(v[u][i][1] & 0xffff0000u), wgt, acc[i][3]);
        }
      }
    }
    const float inv = __builtin_amdgcn_rcpf(lsum);
    CB_GLOBAL uint16_t* orow = gout + grow[rr] * D;
#pragma unroll
    for (int i = 0; i < NDT; i++) {
      uintx2 pk;
      pk[0] = (uint32_t)f2bf(acc[i][0] * inv) | ((uint32_t)f2bf(acc[i][1] * inv) << 16);
      pk[1] = (uint32_t)f2bf(acc[i][2] * inv) | ((uint32_t)f2bf(acc[i][3] * inv) << 16);
      *(CB_GLOBAL uintx2*)(orow + 16 * (dt0 + i) + 4 * kg) = pk;
    }
  }
}

// grid: x = split, y = kv head + Hkv * row tile, z = sequence; block = 256 * G threads.
// A ring stage holds 32*G keys.  With SEQ = false the G wave groups share the 64*R rows of the tile
// and group gi takes keys [32 gi, 32 gi + 32) of every stage (short of rows, long on keys: each SIMD
// still holds two waves whose MFMA, LDS and vector phases overlap; the groups' softmax states are
// combined through LDS at the end).  With SEQ = true every wave owns its own 16*R rows -- the tile
// has 64*R*G rows -- and walks through all G key halves of a stage itself, so K/V is read from HBM
// once for a tile of up to 256 rows.
// `hook` (FUSE only) is the workgroup's share of the logits work; with one row tile per wave there
// are registers to spare and its item is woven into the attention's own waits and barriers (see
// LogitsHook).
template <int R, int G, bool SEQ, bool FUSE, bool TS>
__device__ __forceinline__ void attn_tile(const AttnParams& p_arg, const SeqMetaLanes& ml, unsigned long long ts0,
                                          LogitsHook<256 * G>* hook, unsigned long long* ts_sh) {
  constexpr bool kHookEarly = FUSE && R == 1;
  static_assert(G == 1 || (G == 2 && R <= 2), "two wave groups are built for one or two row tiles per wave");
  constexpr int RT = 64 * R * (SEQ ? G : 1);  // rows of the workgroup's tile
  // All kernel arguments are fetched in one burst at entry (see pin_args): left to itself the
  // compiler loads each near its first use, behind early exits, and the chain of dependent scalar
  // loads then costs several microseconds before the first K/V request goes out.
  AttnParams p = p_arg;
  pin_args(p);
  // (the pinned pointers have lost their address space: say again that they are global memory)
  const CB_GLOBAL uint16_t* gq = (const CB_GLOBAL uint16_t*)p.q;
  CB_GLOBAL uint16_t* gout = (CB_GLOBAL uint16_t*)p.out;
  const CB_GLOBAL char* kbase = (const CB_GLOBAL char*)p.kv.k;
  const CB_GLOBAL char* vbase = (const CB_GLOBAL char*)p.kv.v;
  const CB_GLOBAL int32_t* gbt = (const CB_GLOBAL int32_t*)p.kv.block_table;
  const CB_GLOBAL int32_t* gparent = (const CB_GLOBAL int32_t*)p.parent;
  constexpr int NT = 256 * G;
  static_assert(G == 2, "the ring's requests are shared out among eight waves");
  constexpr int SK = kStageKeys * G;  // keys per stage: two half-stages
  // The ring: NH half-stage slots, each 8 KiB of K followed by 8 KiB of V; half-stage h of the
  // split (keys k0 + 32 h ..) lives in slot h % NH.
  __shared__ uint4 ring[NH * 2 * kStageVecs];
  __shared__ int bt_lds[kMaxBtLds];
  __shared__ AncScratch anc_sh;  // ancestor sets of the whole tree, built here by the splits that reach the tree
  __shared__ int last_flag;
  __shared__ int merge_flag;                 // cooperative merge: thread 64's verdict (0 = not yet)
  __shared__ unsigned long long merge_todo;  // ... and the slices this workgroup merges
  __shared__ int merge_flag2;                // second verdict: slices of workgroups that gave up (completing workgroup only)
  __shared__ unsigned long long merge_todo2;
  constexpr int D = 128;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int gi = w >> 2, wi = w & 3;
  const int c = l & 15, kg = l >> 4;
  // Workgroups are handed to the 8 XCDs round-robin in dispatch order.  With xcd_remap the
  // dispatch index d is renumbered to j = (d % 8) * (T / 8) + d / 8, so that consecutive j --
  // in particular all splits of one (sequence, kv head, row tile) -- sit on the same XCD and
  // meet in its L2.  Tiles are numbered with the sequence running fastest: an XCD's share of the
  // tiles (a contiguous range of j) then holds a few heads of every sequence rather than every
  // head of a few sequences, so a batch of unequal lengths loads the XCDs equally.
  int split, by, b;
  {
    const int T = p.grid_x * p.grid_y * p.grid_z;
    const int d = blockIdx.x + p.grid_x * (blockIdx.y + p.grid_y * blockIdx.z);
    if (p.xcd_remap == 2) {
      // XCD x = d % 8 works through position r = d / 8 of its own list: all splits of a tile together,
      // the tiles of one sequence together, the sequences from the longest to the shortest -- so the
      // workgroups that are dispatched last, and decide when the launch ends, are the short ones.  The
      // XCD's tiles are the same grid_y / 8 (kv head, row tile) pairs of every sequence.
      const int x = d & 7, r = d >> 3;
      split = r % p.grid_x;
      const int tile = r / p.grid_x;
      const int ypx = p.grid_y >> 3;
      by = x * ypx + tile % ypx;
      b = __builtin_amdgcn_readlane(ml.ord, tile / ypx);
    } else {
      const int j = p.xcd_remap ? (d & 7) * (T >> 3) + (d >> 3) : d;
      split = j % p.grid_x;
      const int rest = j / p.grid_x;
      b = rest % p.grid_z;
      by = rest / p.grid_z;
    }
  }
  // (row tiles of one kv head are neighbours in j: they sweep the same K/V and then share an XCD's L2)
  const int tiles = p.grid_y / p.Hkv;
  const int rt = by % tiles, hk = by / tiles;
  const int g = p.Hq / p.Hkv;
  const SeqShape shp = seq_shape(ml, b);
  const int wg_linear = blockIdx.x + p.grid_x * (blockIdx.y + p.grid_y * blockIdx.z);
  // (timing aid: the stamps go to LDS and are copied out when the kernel ends -- a store to memory
  // here, even one that never executes, makes the compiler treat the loads in flight as unordered
  // and wait for all of them wherever it needs one)
  CB_LDS unsigned long long* ts = (CB_LDS unsigned long long*)ts_sh;
  // (TS: the timeline build of the kernel, a measurement aid; every stamp below is compiled out of the
  // kernels that ship as the default)
  const bool do_ts = TS && threadIdx.x == 0 && wg_linear < 1024;
  const bool do_ts64 = TS && threadIdx.x == 64 && wg_linear < 1024;
#define CB_TS(i) do { if (do_ts) ts[i] = wall_clock64(); } while (0)
  if (do_ts) {
#pragma unroll
    for (int i = 1; i < 16; i++) ts[i] = 0;
    ts[0] = ts0;
  }
  CB_TS(1);
  const int off = shp.off, N = shp.N, S = shp.S;
  const int M = N * g;
  const int row0 = rt * RT;
  if (row0 >= M) return;
  const int len = S + N;
  const int k0 = split * p.chunk;
  if (k0 >= len) return;
  const int k1 = (k0 + p.chunk < len) ? k0 + p.chunk : len;
  const int nst = (k1 - k0 + SK - 1) / SK;
  const int nsplit_b = (len + p.chunk - 1) / p.chunk;

  KeyAddr ka;
  ka.kv = &p.kv;
  ka.bt = bt_lds;
  ka.bt_first = 0;
  ka.bs_shift = 0;
  ka.seq = b;
  ka.head = hk;
  if (p.kv.block_size > 0) {  // the launcher guarantees a power-of-two block size and a slice that fits
    ka.bs_shift = 31 - __clz(p.kv.block_size);
    const int first = k0 >> ka.bs_shift, last = (k1 - 1) >> ka.bs_shift;
    for (int i = tid; i <= last - first && i < kMaxBtLds; i += NT)
      bt_lds[i] = gbt[(int64_t)b * p.kv.max_blocks + first + i];
    ka.bt_first = first;
    __syncthreads();  // the K/V addresses below depend on it
  }
  // The workgroup's logits item is requested first of all, into registers.  Loads return in the
  // order of their requests, so wherever these sit they hold up what was requested behind them for
  // as long as they take (cold pages of another buffer); in front of the K/V prologue that time
  // overlaps with the prologue's own first-data latency, and the first stage's wait covers them.
  if constexpr (kHookEarly) hook->prefetch_first();
  // Everything this workgroup needs from memory is requested up front, oldest first: the query rows
  // and ancestor words (to registers), then the whole ring of K/V half-stages (to LDS).
  WaveState<R> st;
  int row_node[R];    // tree node of the lane's query (indexes the ancestor sets)
  int64_t grow[R];    // global output row (node * Hq + head), or -1 past the end
  int nvt = 0;        // this wave's row tiles that hold at least one real row (they come first)
#pragma unroll
  for (int rr = 0; rr < R; rr++) {
    const int rl = ((SEQ ? w : wi) * R + rr) * 16 + c;
    if (row0 + rl - c < M) nvt = rr + 1;
    int row = row0 + rl;
    const bool valid = row < M;
    row = valid ? row : M - 1;
    const int node = row / g, hg = row - node * g;
    row_node[rr] = node;
    const int64_t gr = (int64_t)(off + node) * p.Hq + hk * g + hg;
    grow[rr] = valid ? gr : -1;
    const CB_GLOBAL uintx4* qp = (const CB_GLOBAL uintx4*)(gq + gr * D);
#pragma unroll
    for (int ds = 0; ds < 4; ds++) st.q[rr][ds] = __builtin_bit_cast(bf16x8, load_b128_untracked(qp + kg + 4 * ds));
#pragma unroll
    for (int dt = 0; dt < 8; dt++) st.o[rr][dt] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.lacc[rr] = floatx4{0.f, 0.f, 0.f, 0.f};
    st.mref[rr] = -INFINITY;
  }
  const bool tree_split = k1 > S;  // this split reaches the tree nodes: masks needed
  // the tree itself: one parent entry per thread, requested before the K/V loads
  int my_parent = -1;
  if (tree_split && tid < N && tid < CB_MAX_NODES) {
    if (tid > 0) {
      my_parent = gparent[off + tid];
      if (my_parent < 0 || my_parent >= tid) my_parent = 0;  // (same repair as the acceptance kernel, which reports it)
    }
  }

  const float c2 = p.scale * 1.4426950408889634f;  // softmax scale in the log2 domain
  const int last_key = k1 - 1;  // requests past the split's end repeat its last row (never used; the next split reads its own keys)

  const int nh = (k1 - k0 + kStageKeys - 1) / kStageKeys;  // half-stages of this split
  const int nhw = nh < NH ? NH : nh;                       // half-stages requested
  auto issue = [&](int h, int slot) {
    uint4* const base = ring + slot * (2 * kStageVecs);
    issue_half(base, base + kStageVecs, ka, kbase, vbase, k0 + h * kStageKeys, last_key, w, l);
  };
  // The prologue requests PRO half-stages, and the rest of the ring goes out right behind the
  // first stage's barrier -- all unconditionally (requests past the split's end repeat its last
  // key and are never used), so every wave has a known number of requests behind its query loads,
  // which is what the counted waits below rely on.  (A compute unit takes about 0.3 us to issue a
  // half-stage's requests; with the whole ring in front of the first wait the first stage's
  // arithmetic starts that much later for every half-stage added.)  A split of up to 32 NH keys
  // -- the 7B-shaped workload's 288 -- is thereby requested in full before any of its arithmetic.
#pragma unroll
  for (int h = 0; h < PRO; h++) {
    issue(h, h);
  }
  CB_TS(2);
  if (tree_split) build_ancestor_sets(anc_sh, N, my_parent, jump_rounds(p.max_depth));  // uniform in the workgroup; hidden behind the first K/V wait
  // The first stage's wait, outside the ring loop: it also covers the query loads (older than the
  // whole prologue), whose registers are pinned here.
  wait_vmcnt<2 * (PRO - 2)>();
  ring_barrier();
#pragma unroll
  for (int rr = 0; rr < R; rr++)
#pragma unroll
    for (int ds = 0; ds < 4; ds++) asm volatile("" : "+v"(st.q[rr][ds]));
  CB_TS(3);
  // The logits item rides on the sweep's waits and barriers: its reduction here (its loads are
  // older still than the query's), the combination of the waves' candidates and the partial's
  // store behind the first stage's barrier, the scan ticket at the last stage if that stage's wait
  // is a full one, which then covers that store.
  if constexpr (kHookEarly) hook->mid_consume();

// the row tiles of a wave that lie past the sequence's rows are left out (R = 2: all, one or none)
#define CB_COMPUTE(kp, vp, key0, need_mask)                                                                    \
  do {                                                                                                         \
    if constexpr (R == 2) {                                                                                    \
      if (nvt == R && !(need_mask)) { compute_stage_pair(kp, vp, st, c2, l); break; }                          \
    }                                                                                                          \
    if (nvt == R) compute_stage<R, R>(kp, vp, st, c2, key0, S, k1, need_mask, &anc_sh.anc[0][0], row_node, l);  \
    else if (R > 1) compute_stage<R, 1>(kp, vp, st, c2, key0, S, k1, need_mask, &anc_sh.anc[0][0], row_node, l);\
  } while (0)
  // Stage s = half-stages 2s and 2s+1.  With SEQ = false wave group gi computes half-stage 2s + gi,
  // with SEQ = true every wave computes both.  Each wave issues two requests per half-stage, and
  // requests complete in order, so "at most 2 y requests outstanding" means that everything up to
  // the y youngest half-stages has landed.  At the top of stage s the half-stages requested so far
  // are the prologue's PRO, the rest of the ring (at the top of stage 0) and the refills made at
  // the tops of stages 1 .. s-1.
  int sa = 0;  // ring slot of half-stage 2s
  for (int s = 0; s < nst; s++) {
    const int requested = s == 0 ? PRO : (nhw < 2 * s + NH - 2 ? nhw : 2 * s + NH - 2);
    const int younger = requested - (2 * s + 2);
    static_assert(PRO - 2 <= 5 && NH - 4 <= 5, "the waits below cover up to five younger half-stages");
    if (younger >= 5) wait_vmcnt<10>();
    else if (younger == 4) wait_vmcnt<8>();
    else if (younger == 3) wait_vmcnt<6>();
    else if (younger == 2) wait_vmcnt<4>();
    else if (younger == 1) wait_vmcnt<2>();
    else wait_vmcnt<0>();
    ring_barrier();  // every wave's share of stage s has landed, and nobody reads stage s-1 any more
    const int sb = sa + 1 == NH ? 0 : sa + 1;
    if (s == 0) {
#pragma unroll
      for (int h = PRO; h < NH; h++) issue(h, h);
    } else {  // stage s-1's two slots take the next two half-stages
      const int ha = 2 * s + NH - 2;
      const int ra = sa >= 2 ? sa - 2 : sa - 2 + NH, rb = sa >= 1 ? sa - 1 : sa - 1 + NH;
      if (ha < nh) issue(ha, ra);
      if (ha + 1 < nh) issue(ha + 1, rb);
    }
    if constexpr (kHookEarly) {
      if (s == 0) hook->mid_combine();
      if (s == nst - 1 && younger <= 0) hook->early_ticket();  // behind this stage's vmcnt(0)
    }
#pragma unroll
    for (int h = SEQ ? 0 : gi; h < (SEQ ? G : gi + 1); h++) {
      const int key0 = k0 + (2 * s + h) * kStageKeys;
      const bool need_mask = key0 + kStageKeys > S || key0 + kStageKeys > k1;
      const uint4* const kp = ring + (h == 0 ? sa : sb) * (2 * kStageVecs);
      if (key0 < k1 && nvt > 0) CB_COMPUTE(kp, kp + kStageVecs, key0, need_mask);
    }
    sa = sb + 1 == NH ? 0 : sb + 1;
  }
#undef CB_COMPUTE

  wait_vmcnt<0>();  // (a short split: the unused rest of the prologue must land before the ring is reused)
  CB_TS(4);
  if constexpr (kHookEarly) {
    hook->scan_first();  // its store completes together with the partials' stores below
    hook->stamp(2);
  }

  // With two wave groups each group finishes one half of the head dimension: dim tiles
  // [dt0, dt0 + ndt).  It parks the other half of its accumulators and its (mref, l) in the ring,
  // and adds the partner's parked half to its own.
  constexpr bool kTwoGroups = G == 2 && !SEQ;
  const int dt0 = kTwoGroups ? 4 * gi : 0;
  constexpr int ndt = kTwoGroups ? 4 : 8;
  if constexpr (kTwoGroups) {
    __syncthreads();  // every wave is done with the ring
    const int lane = wi * 64 + l;
    uint4* const park = ring;  // 16 accumulator tiles x 256 lanes x 16 B, then the (mref, l) pairs
    float2* const park_ml = reinterpret_cast<float2*>(ring + 16 * 256);
    // (the group index is a compile-time constant inside, so that ring slots and accumulators keep
    // constant indices)
    auto park_half = [&](auto gic) {
      constexpr int GI = decltype(gic)::value;
#pragma unroll
      for (int rr = 0; rr < R; rr++) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int dt = 4 * (1 - GI) + i;  // the partner's half
          const int slot = rr * 8 + dt;
          park[slot * 256 + lane] = __builtin_bit_cast(uint4, st.o[rr][dt]);
        }
        park_ml[(GI * R + rr) * 256 + lane] = float2{st.mref[rr], st.lacc[rr][0]};
      }
    };
    auto take_half = [&](auto gic) {
      constexpr int GI = decltype(gic)::value;
#pragma unroll
      for (int rr = 0; rr < R; rr++) {
        const float2 ml2 = park_ml[((1 - GI) * R + rr) * 256 + lane];
        const float m = fmaxf(st.mref[rr], ml2.x);
        const float mu = (m == -INFINITY) ? 0.f : m;
        const float w0 = __builtin_amdgcn_exp2f((st.mref[rr] - mu) * c2), w1 = __builtin_amdgcn_exp2f((ml2.x - mu) * c2);
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int dt = 4 * GI + i;
          const int slot = rr * 8 + dt;
          const floatx4 a = __builtin_bit_cast(floatx4, park[slot * 256 + lane]);
          st.o[rr][dt] = st.o[rr][dt] * w0 + a * w1;
        }
        st.lacc[rr][0] = st.lacc[rr][0] * w0 + ml2.y * w1;
        st.mref[rr] = m;
      }
    };
    if (gi == 0) park_half(std::integral_constant<int, 0>{}); else park_half(std::integral_constant<int, 1>{});
    __syncthreads();
    if (gi == 0) take_half(std::integral_constant<int, 0>{}); else take_half(std::integral_constant<int, 1>{});
  }

  if constexpr (kHookEarly) hook->stamp(3);
  // Buffer descriptor over this sequence's partials (byte offsets fit 32 bits, checked by the launcher).
  const __amdgpu_buffer_rsrc_t prsrc = __builtin_amdgcn_make_buffer_rsrc(
      reinterpret_cast<char*>(p.partial) + unit_tile0(off, p.Hq, p.Hkv, b) * p.nsplit * kUnitBytes, 0, 0x7fffffff, 0x00020000);
  uint32_t ubyte[R];  // split 0's unit of each of this wave's row tiles
#pragma unroll
  for (int rr = 0; rr < R; rr++) {
    const int ti = (row0 >> 4) + (SEQ ? w : wi) * R + rr;
    ubyte[rr] = (uint32_t)(hk * ((M + 15) >> 4) + ti) * (uint32_t)p.nsplit * (uint32_t)kUnitBytes;
  }
  // finish.  Every lane holds its query's full denominator.
  {
#pragma unroll
    for (int rr = 0; rr < R; rr++) {
      const float lt = st.lacc[rr][0];
      if (grow[rr] < 0) continue;
      if (nsplit_b == 1) {
        const float inv = 1.0f / lt;
        CB_GLOBAL uint16_t* orow = gout + grow[rr] * D;
#pragma unroll
        for (int i = 0; i < ndt; i++) {
          const floatx4 o = (kTwoGroups && gi == 1) ? st.o[rr][(4 + i) & 7] : st.o[rr][i];
          const int dt = dt0 + i;
          uintx2 pk;
          pk[0] = (uint32_t)f2bf(o[0] * inv) | ((uint32_t)f2bf(o[1] * inv) << 16);
          pk[1] = (uint32_t)f2bf(o[2] * inv) | ((uint32_t)f2bf(o[3] * inv) << 16);
          *(CB_GLOBAL uintx2*)(orow + 16 * dt + 4 * kg) = pk;
        }
      } else {
        // partial state of this split, written through to memory (agent scope) so that the merging
        // workgroup, possibly on another XCD with its own L2, can read it without cache flushes
        const uint32_t pbyte = ubyte[rr] + (uint32_t)split * kUnitBytes;
#pragma unroll
        for (int i = 0; i < ndt; i++) {
          const floatx4 o = (kTwoGroups && gi == 1) ? st.o[rr][(4 + i) & 7] : st.o[rr][i];
          const int dt = dt0 + i;
          const uintx2 v = {(uint32_t)f2bf(o[0]) | ((uint32_t)f2bf(o[1]) << 16),
                            (uint32_t)f2bf(o[2]) | ((uint32_t)f2bf(o[3]) << 16)};
          if (p.external_merge) __builtin_amdgcn_raw_buffer_store_b64(v, prsrc, pbyte + dt * 512 + l * 8, 0, 0);
          else __builtin_amdgcn_raw_buffer_store_b64(v, prsrc, pbyte + dt * 512 + l * 8, 0, kAgentCoherent);
        }
        if (kg == 0 && (!kTwoGroups || gi == 0)) {
          // m = log2 of the reference weight 2^(c2*mref)
          const float mnat = (st.mref[rr] == -INFINITY) ? -INFINITY : st.mref[rr] * c2;  // log2 units
          const uintx2 ml = {__float_as_uint(mnat), __float_as_uint(lt)};
          if (p.external_merge) __builtin_amdgcn_raw_buffer_store_b64(ml, prsrc, pbyte + kUnitMl + c * 8, 0, 0);
          else __builtin_amdgcn_raw_buffer_store_b64(ml, prsrc, pbyte + kUnitMl + c * 8, 0, kAgentCoherent);
        }
      }
    }
  }
  if constexpr (kHookEarly) hook->stamp(4);
  if (nsplit_b == 1 || p.external_merge) return;  // (a following kernel merges: the kernel boundary orders the stores)

  // ---- split merge.  The partials above are write-through stores; once they have completed
  // (vmcnt 0) the workgroup takes a ticket with a device-scope atomic.  No cache-wide write-back or
  // invalidate is involved (a __threadfence() per workgroup costs a full L2 sweep on this chip).
  //
  // Ticket word of a tile (64 bits, zero between launches): arrivals in bits 0-11 and, to learn
  // whether every split ran on one XCD, the sum (bits 24-39) and the sum of squares (bits 40-59)
  // of the arrivals' XCC_ID (hardware register 20, bits 3:0): all ids equal mine  <=>
  // sum = n*id and sumsq = n*id*id.  A second word per tile holds one bit per split whose
  // workgroup gave up waiting (cooperative merge only).
  if (tid == 64) { merge_flag = 0; merge_flag2 = 0; }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  CB_TS(5);
  // (cooperative merge: the tiles' words are polled, so each tile has a 4 KiB stretch of its own
  // in a separate area -- neighbours in one line would all be served by one memory channel)
  const int64_t tile_id = ((int64_t)b * p.Hkv + hk) * tiles + rt;
  CB_GLOBAL unsigned long long* ticket = p.coop_merge ? (CB_GLOBAL unsigned long long*)p.coop_tickets + tile_id * (kCoopTicketStride / 8)
                                                      : (CB_GLOBAL unsigned long long*)p.tickets + 2 * tile_id;
  constexpr unsigned long long kArrivals = 0xfffull;
  const unsigned long long xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & 15u;
  const unsigned long long arrive = 1ull | (xcc << 24) | ((xcc * xcc) << 40);
  auto one_xcd = [&](unsigned long long tot) {
    const unsigned long long n = tot & kArrivals, sum = (tot >> 24) & 0xffffull, sumsq = tot >> 40;
    return sum == n * xcc && sumsq == n * xcc * xcc;
  };

  if (!p.coop_merge) {
    // Merge by the last workgroup of the tile to arrive: the others leave at once and free their
    // compute units (grids of several rounds of workgroups).
    if (tid == 0) {
      uint32_t scan_old = 0;
      if constexpr (kHookEarly) scan_old = hook->ticket_first_issue();
      const unsigned long long tot = __hip_atomic_fetch_add(ticket, arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + arrive;
      int flag = ((tot & kArrivals) == (unsigned long long)nsplit_b) ? 1 : 0;
      if (flag) {
        if (!one_xcd(tot)) {
          flag = 2;  // some split ran on another XCD: its partials are not in this L2
          __hip_atomic_fetch_or((CB_GLOBAL int32_t*)p.status, 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __hip_atomic_store(ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
      }
      last_flag = flag;
      if constexpr (kHookEarly) hook->ticket_first_resolve(scan_old);
    }
    __syncthreads();
    CB_TS(6);
    // If this workgroup completed the logits scan, its first wave runs the acceptance now, while the
    // other waves go straight on to the merge below.
    if constexpr (kHookEarly) {
      hook->first_counted();
      hook->accept_first();
      hook->stamp(5);
    }
    if (!last_flag) return;
    // Same XCD: the write-through stores left the lines in this L2, plain (cached) loads are coherent
    // with them.  Otherwise read past the L2 with agent-coherent loads.
    if (last_flag == 1) merge_tile<R, ndt, 0>(prsrc, grow, ubyte, gout, nsplit_b, dt0, l);
    else merge_tile<R, ndt, kAgentCoherent>(prsrc, grow, ubyte, gout, nsplit_b, dt0, l);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    CB_TS(7);
    return;
  }

  // ---- cooperative merge (the whole grid is resident at once: one round of workgroups).  Every
  // workgroup of the tile merges a slice of it -- the (16-row tile, dim tile) units u with
  // u % nsplit_b == split -- once all splits have arrived, so no compute unit has to pull the whole
  // tile's partials through its own memory pipe.  Thread 64 arrives and then polls the ticket, at
  // most spin_limit times: the tile is complete when the arrivals equal nsplit_b, or when the word
  // is zero again (the completing workgroup zeroes it for the next launch; after one's own arrival
  // it cannot be zero for any other reason).  A workgroup that gives up sets its bit in the tile's
  // second word, looks at the ticket once more and leaves if the tile is still incomplete: the
  // completing workgroup reads that word after its own arrival, so it finds the bit and merges the
  // slice.  (If the last look shows the tile complete after all, the workgroup merges its slice
  // itself: the completing workgroup may have read the word before the bit was there.  If both
  // merge it they write the same bytes.)  Wave 0 is not waited for by anyone: in the one-launch
  // verification it draws the logits ticket and may have to run the acceptance first.
  CB_GLOBAL unsigned long long* gave_up = ticket + 1;
  if constexpr (kHookEarly) {
    if (tid == 0) hook->ticket_first_resolve(hook->ticket_first_issue());
    hook->first_counted();
    hook->accept_first();
    hook->stamp(5);
  }
  if (tid == 64) {
    unsigned long long tot = __hip_atomic_fetch_add(ticket, arrive, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + arrive;
    const bool completes = (tot & kArrivals) == (unsigned long long)nsplit_b;
    auto complete = [&](unsigned long long t) { return (t & kArrivals) == (unsigned long long)nsplit_b || t == 0ull; };
    for (int spin = 0; !complete(tot) && spin < p.spin_limit; spin++) {
      __builtin_amdgcn_s_sleep(2);
      tot = __hip_atomic_load(ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    unsigned long long todo = 1ull << split, todo2 = 0;
    bool own_bit = false;
    if (!complete(tot)) {
      // (the returning form: the bit is in memory before the ticket is looked at again)
      const unsigned long long before = __hip_atomic_fetch_or(gave_up, 1ull << split, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      asm volatile("s_waitcnt vmcnt(0)" ::"v"(before) : "memory");
      tot = __hip_atomic_load(ticket, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      own_bit = true;
      if (!complete(tot)) todo = 0;
      __hip_atomic_fetch_or((CB_GLOBAL int32_t*)p.status, 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // plain loads only when the ticket itself says that every split ran on this XCD
    int flag = (tot != 0ull && one_xcd(tot)) ? 1 : 2;
    if (todo != 0 && flag == 2) __hip_atomic_fetch_or((CB_GLOBAL int32_t*)p.status, 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    merge_todo = todo;
    __hip_atomic_store(&merge_flag, flag, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    if (do_ts64) ts[6] = wall_clock64();
    if (completes) {
      todo2 = __hip_atomic_load(gave_up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) & ~todo;
      if (todo2 != 0) __hip_atomic_store(gave_up, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(ticket, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    } else if (own_bit && todo != 0) {
      __hip_atomic_fetch_and(gave_up, ~(1ull << split), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    merge_todo2 = todo2;
    __hip_atomic_store(&merge_flag2, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
  }
  // Unit u of the tile = (16-row tile u / 8, dim tile u % 8); this workgroup's own slice holds the
  // units split, split + nsplit_b, ...; its k-th unit goes to wave (k + 1) % NW.  What a wave needs
  // for its first unit -- the lane's output row, the partials' offsets -- is worked out before it
  // waits, so that the loads go out as soon as the verdict is in.
  constexpr int NW = NT / 64;
  constexpr int NU = (RT / 16) * 8;
  const int nslots = nsplit_b;
  auto unit_row = [&](int u, int64_t* gr, uint32_t* ub) {  // false: no rows in this unit's tile
    const int tl = u >> 3;
    const int row = row0 + tl * 16 + c;
    if (row - c >= M) return false;
    const int node = row / g, hg = row - node * g;
    *gr = row < M ? (int64_t)(off + node) * p.Hq + hk * g + hg : -1;
    *ub = (uint32_t)(hk * ((M + 15) >> 4) + (row0 >> 4) + tl) * (uint32_t)p.nsplit * (uint32_t)kUnitBytes;
    return true;
  };
  auto merge_one = [&](int u, int64_t gr, uint32_t ub, int flag) {
    int64_t gr1[1] = {gr};
    uint32_t ub1[1] = {ub};
    const int dt = u & 7;
    if (nslots <= 8) {  // (one batch in the common cases)
      if (flag == 1) merge_tile<1, 1, 0, 8>(prsrc, gr1, ub1, gout, nslots, dt, l);
      else merge_tile<1, 1, kAgentCoherent, 8>(prsrc, gr1, ub1, gout, nslots, dt, l);
    } else {
      if (flag == 1) merge_tile<1, 1, 0, 16>(prsrc, gr1, ub1, gout, nslots, dt, l);
      else merge_tile<1, 1, kAgentCoherent, 16>(prsrc, gr1, ub1, gout, nslots, dt, l);
    }
  };
  const int u_first = split + ((w + NW - 1) % NW) * nsplit_b;  // this wave's first unit of the own slice
  int64_t gr_first = -1;
  uint32_t ub_first = 0;
  const bool have_first = u_first < NU && unit_row(u_first, &gr_first, &ub_first);
  // the waves wait for thread 64's verdicts in LDS (no barrier: wave 0 may still be busy)
  int flag;
  while ((flag = __hip_atomic_load(&merge_flag, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP)) == 0) __builtin_amdgcn_s_sleep(1);
  if (do_ts64) ts[8] = wall_clock64();
  auto merge_slices = [&](unsigned long long todo, bool first_done) {
    int k = 0;  // running number of the units of the slices in `todo`
    for (int s2 = 0; s2 < nsplit_b; s2++) {
      if (!((todo >> s2) & 1ull)) continue;
      for (int u = s2; u < NU; u += nsplit_b, k++) {
        if ((k + 1) % NW != w || (first_done && u == u_first)) continue;
        int64_t gr;
        uint32_t ub;
        if (unit_row(u, &gr, &ub)) merge_one(u, gr, ub, flag);
      }
    }
  };
  const unsigned long long todo1 = merge_todo;
  if (todo1 == (1ull << split)) {  // the usual case: the own slice
    if (have_first) merge_one(u_first, gr_first, ub_first, flag);
    if (u_first + NW * nsplit_b < NU) merge_slices(todo1, true);
  } else if (todo1 != 0) {
    merge_slices(todo1, false);
  }
  if (do_ts64) ts[9] = wall_clock64();

  while (__hip_atomic_load(&merge_flag2, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) == 0) __builtin_amdgcn_s_sleep(1);
  if (merge_todo2 != 0) merge_slices(merge_todo2, false);
  if (do_ts64) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    ts[7] = wall_clock64();
  }
#undef CB_TS
}

// Timing aid (timeline build): thread 0 copies the workgroup's stamps from LDS to the table, the
// attention's eight to row wg, the logits hook's eight to row wg + 512.
template <bool TS>
__device__ __forceinline__ void flush_timestamps(const AttnParams& p, const unsigned long long* ts_sh, bool hook_rows) {
  if constexpr (!TS) return;
  const int wg = blockIdx.x + p.grid_x * (blockIdx.y + p.grid_y * blockIdx.z);
  __syncthreads();  // (thread 64 stamps too)
  if (threadIdx.x != 0 || wg >= 1024) return;
  const CB_LDS unsigned long long* ts = (const CB_LDS unsigned long long*)ts_sh;
  CB_GLOBAL unsigned long long* out = (CB_GLOBAL unsigned long long*)p.dbg_ts;
  for (int i = 0; i < 8; i++) out[(int64_t)wg * 8 + i] = ts[i];
  if (hook_rows && wg < 512)
    for (int i = 0; i < 8; i++) out[(int64_t)(wg + 512) * 8 + i] = ts[8 + i];
}

template <int R, int G, bool SEQ, bool TS>
__global__ __launch_bounds__(256 * G) void k_attn_mfma(AttnParams p, SeqMeta meta) {
  const unsigned long long ts0 = TS ? wall_clock64() : 0ull;
  const SeqMetaLanes ml = seq_meta_prefetch(meta);
  __shared__ unsigned long long ts_sh[TS ? 16 : 1];
  attn_tile<R, G, SEQ, false, TS>(p, ml, ts0, nullptr, ts_sh);
  flush_timestamps<TS>(p, ts_sh, true);
}

// The whole verification in one launch: every workgroup does its attention duty (a tile's split,
// perhaps the tile's merge) and takes its share of the logits scan; the workgroup that completes a
// sequence's scan runs the sequence's acceptance (LogitsHook of cb_logits.h).  The scan does not
// depend on the attention, so it needs no ordering against it, and its memory round trips ride on
// those the attention needs anyway.
template <int R, int G, bool SEQ, bool TS>
__global__ __launch_bounds__(256 * G) void k_verify_mfma(AttnParams p, SeqMeta meta, LogitsWork lw_arg) {
  const unsigned long long ts0 = TS ? wall_clock64() : 0ull;
  const SeqMetaLanes ml = seq_meta_prefetch(meta);
  LogitsWork lw = lw_arg;
  pin_logits_args(lw);  // fetched with the attention's arguments, not later in front of the first use
  __shared__ TailLds tail;
  const int wg = blockIdx.x + p.grid_x * (blockIdx.y + p.grid_y * blockIdx.z);
  LogitsHook<256 * G> hook(lw, ml, tail, wg);
  __shared__ unsigned long long ts_sh[TS ? 16 : 1];
  if constexpr (TS) hook.dbg = (CB_LDS unsigned long long*)ts_sh + 8;  // (timing aid)
  attn_tile<R, G, SEQ, true, TS>(p, ml, ts0, &hook, ts_sh);
  hook.finish();
  flush_timestamps<TS>(p, ts_sh, true);
}

// Stand-alone merge of the bf16 partials, used when a tile's partials are too many for one
// workgroup to pull through its compute unit: one workgroup per 16-row tile, its four waves take two
// dim tiles each; lane (kg, c) -> row c, dims 16 dt + 4 kg + {0..3}, as the partials are laid out.
// grid: x = 16-row tile, y = kv head, z = sequence; block = 256 threads.
__global__ __launch_bounds__(256) void k_merge_partials_bf16(AttnParams p, SeqMeta meta) {
  constexpr int D = 128;
  constexpr int NDT = 2;
  const int l = threadIdx.x & 63, c = l & 15, kg = l >> 4;
  const int dt0 = (threadIdx.x >> 6) * NDT;
  const int b = blockIdx.z, hk = blockIdx.y, ti = blockIdx.x;
  const int g = p.Hq / p.Hkv;
  const int off = meta.node_off[b], N = meta.node_off[b + 1] - off;
  const int M = N * g;
  const int row = ti * 16 + c;
  if (row >= M) return;
  const int len = meta.kv_len[b] + N;
  const int ns = (len + p.chunk - 1) / p.chunk;
  if (ns <= 1) return;  // the attention kernel already wrote the output
  const char* pr = reinterpret_cast<const char*>(p.partial) +
                   (unit_tile0(off, p.Hq, p.Hkv, b) + (int64_t)hk * ((M + 15) >> 4) + ti) * p.nsplit * kUnitBytes;
  floatx4 acc[NDT];
#pragma unroll
  for (int i = 0; i < NDT; i++) acc[i] = floatx4{0.f, 0.f, 0.f, 0.f};
  float lsum = 0.f, m_run = -3.0e38f;  // (kept finite: a slot without a visible key carries m = -inf and gets weight 0)
  constexpr int BS = 8;
  for (int t0 = 0; t0 < ns; t0 += BS) {
    uint2 v[BS][NDT];
    float2 ml[BS];
#pragma unroll
    for (int u = 0; u < BS; u++) {
      const int t = (t0 + u < ns) ? t0 + u : ns - 1;
      const char* tb = pr + (int64_t)t * kUnitBytes;
      ml[u] = *reinterpret_cast<const float2*>(tb + kUnitMl + c * 8);
#pragma unroll
      for (int i = 0; i < NDT; i++) v[u][i] = *reinterpret_cast<const uint2*>(tb + (dt0 + i) * 512 + l * 8);
    }
    __builtin_amdgcn_sched_barrier(0);  // (every load of the batch requested before the first result is looked at)
    float m_new = m_run;
#pragma unroll
    for (int u = 0; u < BS; u++) m_new = fmaxf(m_new, ml[u].x);
    const float resc = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
    for (int i = 0; i < NDT; i++) acc[i] *= resc;
    lsum *= resc;
    m_run = m_new;
#pragma unroll
    for (int u = 0; u < BS; u++) {
      float wgt = __builtin_amdgcn_exp2f(ml[u].x - m_new);  // m is stored in log2 units
      wgt = (t0 + u < ns) ? wgt : 0.f;
      lsum = fmaf(ml[u].y, wgt, lsum);
#pragma unroll
      for (int i = 0; i < NDT; i++) {
        acc[i][0] = fmaf(__uint_as_float(v[u][i].x << 16), wgt, acc[i][0]);
        acc[i][1] = fmaf(__uint_as_float(v[u][i].x & 0xffff0000u), wgt, acc[i][1]);
        acc[i][2] = fmaf(__uint_as_float(v[u][i].y << 16), wgt, acc[i][2]);
        acc[i][3] = fmaf(__uint_as_float(v[u][i].y & 0xffff0000u), wgt, acc[i][3]);
      }
    }
  }
  const float inv = __builtin_amdgcn_rcpf(lsum);
  const int node = row / g, hg = row - node * g;
  uint16_t* orow = reinterpret_cast<uint16_t*>(p.out) + ((int64_t)(off + node) * p.Hq + hk * g + hg) * D;
#pragma unroll
  for (int i = 0; i < NDT; i++) {
    uint2 pk;
    pk.x = (uint32_t)f2bf(acc[i][0] * inv) | ((uint32_t)f2bf(acc[i][1] * inv) << 16);
    pk.y = (uint32_t)f2bf(acc[i][2] * inv) | ((uint32_t)f2bf(acc[i][3] * inv) << 16);
    *reinterpret_cast<uint2*>(orow + 16 * (dt0 + i) + 4 * kg) = pk;
  }
}

size_t attn_mfma_partial_bytes(size_t max_total_nodes, int Hq, int Hkv, int max_batch, int max_splits) {
  // the last sequence's units end at or before tile max_total_nodes * Hq / 16 + (Hkv + 1) * max_batch
  const size_t tiles = max_total_nodes * Hq / 16 + (size_t)(Hkv + 1) * max_batch + 1;
  return tiles * (size_t)max_splits * kUnitBytes;
}

bool attn_mfma_supports(const AttnParams& p) {
  if (p.D != 128) return false;
  if (p.kv.block_size > 0) {
    if (p.kv.block_size & (p.kv.block_size - 1)) return false;
    if (p.chunk / p.kv.block_size + 2 > kMaxBtLds) return false;
  }
  if (p.nsplit > 4096) return false;  // the ticket counts arrivals in 16 bits
  // partial offsets inside one sequence are 32-bit byte offsets of a buffer descriptor
  if ((int64_t)p.Hkv * ((CB_MAX_NODES * (p.Hq / p.Hkv) + 15) / 16) * p.nsplit * kUnitBytes >= (1ll << 31)) return false;
  return true;
}

// Rows per workgroup tile the launcher picks for a call whose largest sequence has `mrows` rows
// (g query heads x N nodes) per kv head.
int attn_mfma_tile_rows(int mrows) { return mrows <= 64 ? 64 : (mrows <= 128 ? 128 : 256); }

// Whether the launch for this call can also carry the logits work (k_verify_mfma).  That pays when
// each workgroup gets at most one logits item and has registers to hold it during the key sweep:
// the variant with one row tile per wave (so every sequence has at most 64 nodes), no more items
// than workgroups, bf16 logits.  Larger calls run in several rounds of workgroups, where a
// stand-alone scan at full occupancy is faster.
bool attn_mfma_can_fuse(const AttnParams& p, int max_nodes_in_call, int64_t logits_items, int logits_dtype) {
  if (!attn_mfma_supports(p) || logits_dtype != CB_BF16) return false;
  const int M = max_nodes_in_call * (p.Hq / p.Hkv);
  if (attn_mfma_tile_rows(M) != 64) return false;
  const int64_t T = (int64_t)p.nsplit * p.Hkv * p.batch;
  return logits_items <= T;
}

hipError_t launch_attn_mfma(hipStream_t st, const AttnParams& p, const SeqMeta& meta, int max_nodes_in_call,
                            int total_nodes, const LogitsWork* logits_work, int* merge_kind) {
  if (!attn_mfma_supports(p)) return hipErrorInvalidValue;
  const int g = p.Hq / p.Hkv;
  const int M = max_nodes_in_call * g;
  const int rt_rows = attn_mfma_tile_rows(M);
  const int tiles = (M + rt_rows - 1) / rt_rows;
  dim3 grid(p.nsplit, p.Hkv * tiles, p.batch);
  AttnParams q = p;
  const int64_t T = (int64_t)p.nsplit * p.Hkv * tiles * p.batch;
  // renumbering needs whole groups of splits inside each XCD's share of the grid
  q.xcd_remap = (T % 8 == 0 && (T / 8) % p.nsplit == 0) ? 1 : 0;
  if (grid.y % 8 == 0 && p.batch > 1) q.xcd_remap = 2;  // (several sequences: longest first within every XCD)
  q.grid_x = grid.x;
  q.grid_y = grid.y;
  q.grid_z = grid.z;
  // one workgroup can pull about 50 GB/s of partials through its compute unit: beyond a few hundred
  // KiB per tile a separate, fully parallel merge kernel is cheaper than the in-kernel merge
  q.external_merge = (p.nsplit > 1 && (int64_t)p.nsplit * (rt_rows / 16) * kUnitBytes > 320 * 1024) ? 1 : 0;
  // A grid that is resident in one round (one workgroup per compute unit) merges cooperatively:
  // every workgroup of a tile takes a slice, so the volume per compute unit does not grow with
  // the split count and no second launch is needed.
  static int compute_units = 0;
  if (compute_units == 0) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) compute_units = n;
    else compute_units = -1;
  }
  q.coop_merge = (p.coop_merge >= 0 && p.coop_tickets && p.nsplit > 1 && p.nsplit <= 64 && compute_units > 0 && T <= compute_units &&
                  (int64_t)p.Hkv * tiles * p.batch <= kCoopTiles) ? 1 : 0;
  if (q.coop_merge) q.external_merge = 0;
  if (p.force_external_merge && p.nsplit > 1) { q.external_merge = 1; q.coop_merge = 0; }  // (option "external_merge": a test aid)
  if (merge_kind) *merge_kind = p.nsplit <= 1 ? 0 : (q.coop_merge ? 1 : (q.external_merge ? 3 : 2));
  const bool ts = p.timeline != 0;  // (the timeline build of the same kernels: a measurement aid)
#define CB_LAUNCH_ATTN(R, G, SEQ)                                                                           \
  do {                                                                                                      \
    if (ts) hipLaunchKernelGGL((k_attn_mfma<R, G, SEQ, true>), grid, dim3(256 * G), 0, st, q, meta);        \
    else hipLaunchKernelGGL((k_attn_mfma<R, G, SEQ, false>), grid, dim3(256 * G), 0, st, q, meta);          \
  } while (0)
  if (logits_work) {
    const LogitsWork& lw = *logits_work;
    if (!attn_mfma_can_fuse(p, max_nodes_in_call, (int64_t)lw.rows * lw.accept.nchunks, CB_BF16)) return hipErrorInvalidValue;
    if (ts) hipLaunchKernelGGL((k_verify_mfma<1, 2, false, true>), grid, dim3(512), 0, st, q, meta, lw);
    else hipLaunchKernelGGL((k_verify_mfma<1, 2, false, false>), grid, dim3(512), 0, st, q, meta, lw);
  } else if (rt_rows == 64) {
    CB_LAUNCH_ATTN(1, 2, false);
  } else if (rt_rows == 128) {
    CB_LAUNCH_ATTN(2, 2, false);
  } else {
    CB_LAUNCH_ATTN(2, 2, true);
  }
#undef CB_LAUNCH_ATTN
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (q.external_merge) {
    const int tiles16 = (M + 15) / 16;
    hipLaunchKernelGGL(k_merge_partials_bf16, dim3(tiles16, p.Hkv, p.batch), dim3(256), 0, st, q, meta);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace cb

// Device check of an assumption the MFMA attention kernel's load pipeline rests on: vector memory
// loads are counted off vmcnt in the order they were requested, whether they return to registers
// or, as LDS-DMA, to LDS.  The kernel issues both kinds as instructions the compiler does not track
// and covers them with counted waits of its own (cb_attn_mfma.hip); this probe lets a test see the
// order on the machine it runs on.  Every access is in bounds and nothing that needs a wait goes
// without one: the only early read is of a register (or LDS word) that holds a sentinel until its
// load lands.  gfx950 only.
#include <hip/hip_runtime.h>

#include "cacheback.h"

namespace {

#define CB_GLOBAL __attribute__((address_space(1)))
#define CB_LDS __attribute__((address_space(3)))
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kSentinel = 0xdeadbeefu;
constexpr int kStrideDw = 4096;  // 16 KiB between a workgroup's successive cold accesses

__device__ __forceinline__ void lds_dma_b128(const CB_GLOBAL char* src, CB_LDS u32x4* dst) {
  const uint32_t base = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory");
}

// One cold register load, then eight LDS-DMA requests for hot lines.  After "at most 8 requests in
// flight" the register must hold the loaded value.  CONTROL waits for nothing (vmcnt 9) and is
// expected to see the sentinel: it shows that the probe can tell the difference.
template <bool CONTROL>
__global__ __launch_bounds__(64) void k_probe_reg_then_dma(const uint32_t* cold, const uint32_t* hot, uint32_t* result, int iters) {
  __shared__ u32x4 buf[64 * 8];
  const int l = threadIdx.x;
  const CB_GLOBAL uint32_t* gc = (const CB_GLOBAL uint32_t*)cold;
  const CB_GLOBAL char* gh = (const CB_GLOBAL char*)hot;
  uint32_t early_bad = 0, late_bad = 0;
  for (int it = 0; it < iters; it++) {
    const size_t idx = ((size_t)blockIdx.x * iters + it) * kStrideDw + l;
    uint32_t r = kSentinel;
    asm volatile("global_load_dword %0, %1, off" : "+v"(r) : "v"(gc + idx) : "memory");
#pragma unroll
    for (int i = 0; i < 8; i++) lds_dma_b128(gh + l * 16, (CB_LDS u32x4*)buf + i * 64);
    uint32_t early;
    if (CONTROL) asm volatile("s_waitcnt vmcnt(9)\n\tv_mov_b32 %0, %1" : "=v"(early) : "v"(r) : "memory");
    else asm volatile("s_waitcnt vmcnt(8)\n\tv_mov_b32 %0, %1" : "=v"(early) : "v"(r) : "memory");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    asm volatile("" : "+v"(r));
    const uint32_t expect = (uint32_t)idx * 2654435761u + 12345u;
    early_bad += early != expect;
    late_bad += r != expect;
    __syncthreads();
  }
  atomicAdd(&result[CONTROL ? 4 : 0], early_bad);
  atomicAdd(&result[CONTROL ? 5 : 1], late_bad);
}

// The other way round: one cold LDS-DMA request, then eight register loads of hot lines.
__global__ __launch_bounds__(64) void k_probe_dma_then_reg(const uint32_t* cold, const uint32_t* hot, uint32_t* result, int iters) {
  __shared__ u32x4 buf[64];
  const int l = threadIdx.x;
  const CB_GLOBAL char* gc = (const CB_GLOBAL char*)cold;
  const CB_GLOBAL uint32_t* gh = (const CB_GLOBAL uint32_t*)hot;
  uint32_t early_bad = 0, late_bad = 0;
  for (int it = 0; it < iters; it++) {
    const size_t idx = ((size_t)blockIdx.x * iters + it) * kStrideDw + l * 4;
    buf[l] = u32x4{kSentinel, kSentinel, kSentinel, kSentinel};
    __syncthreads();
    lds_dma_b128(gc + idx * 4, (CB_LDS u32x4*)buf);
    uint32_t h[8];
#pragma unroll
    for (int i = 0; i < 8; i++) asm volatile("global_load_dword %0, %1, off" : "=v"(h[i]) : "v"(gh + l + 64 * i) : "memory");
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    const u32x4 early = buf[l];
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    const u32x4 late = buf[l];
#pragma unroll
    for (int i = 0; i < 8; i++) asm volatile("" ::"v"(h[i]));
    const uint32_t expect = (uint32_t)idx * 2654435761u + 12345u;
    early_bad += early.x != expect;
    late_bad += late.x != expect;
    __syncthreads();
  }
  atomicAdd(&result[2], early_bad);
  atomicAdd(&result[3], late_bad);
}

// A plain streaming read: every thread folds 16-byte pieces, eight loads in flight, a grid-stride
// loop; one word per workgroup goes to the sink so that nothing is optimised away.
__global__ __launch_bounds__(512) void k_probe_stream_read(const uint4* __restrict__ src, int64_t n16, uint32_t* sink) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  uint32_t acc = 0;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; u++) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const uint4 v = src[i];
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9e3779b9u) sink[blockIdx.x & 255] = acc;  // (practically never: the loads just have to happen)
}

}  // namespace

extern "C" int cb_probe_stream_read(void* hip_stream, const void* d_src, int64_t bytes, uint32_t* d_sink) {
  if (!d_src || !d_sink || bytes < 16 || (bytes & 15) || ((uintptr_t)d_src & 15)) return CB_EINVAL;
  hipLaunchKernelGGL(k_probe_stream_read, dim3(1024), dim3(512), 0, (hipStream_t)hip_stream,
                     static_cast<const uint4*>(d_src), bytes / 16, d_sink);
  return hipGetLastError() == hipSuccess ? CB_OK : CB_EHIP;
}

extern "C" int cb_probe_load_order(void* hip_stream, const uint32_t* d_cold, int64_t cold_dwords, const uint32_t* d_hot,
                                   int64_t hot_dwords, int32_t workgroups, int32_t iters, uint32_t* d_result) {
  if (!d_cold || !d_hot || !d_result || workgroups < 1 || iters < 1) return CB_EINVAL;
  // the last cold access: ((workgroups*iters - 1) * stride + 63 * 4 + 3) dwords; the hot ones: 512 dwords
  if ((int64_t)workgroups * iters * kStrideDw + 256 > cold_dwords || hot_dwords < 512) return CB_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(k_probe_reg_then_dma<false>, dim3(workgroups), dim3(64), 0, st, d_cold, d_hot, d_result, iters);
  hipLaunchKernelGGL(k_probe_reg_then_dma<true>, dim3(workgroups), dim3(64), 0, st, d_cold, d_hot, d_result, iters);
  hipLaunchKernelGGL(k_probe_dma_then_reg, dim3(workgroups), dim3(64), 0, st, d_cold, d_hot, d_result, iters);
  return hipGetLastError() == hipSuccess ? CB_OK : CB_EHIP;
}

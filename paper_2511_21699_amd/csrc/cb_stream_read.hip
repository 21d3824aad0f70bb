// A plain streaming read, the benchmark's yardstick: what this machine delivers for one launch
// that only reads as many bytes as the attention sweeps.  Not part of the method.  gfx950 only.
#include <hip/hip_runtime.h>

#include "cacheback.h"

namespace {

// grid-stride 16-byte loads, eight in flight per thread, nothing else
__global__ __launch_bounds__(512) void k_stream_read(const uint4* __restrict__ src, int64_t n16, uint32_t* sink) {
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
  hipLaunchKernelGGL(k_stream_read, dim3(1024), dim3(512), 0, (hipStream_t)hip_stream,
                     static_cast<const uint4*>(d_src), bytes / 16, d_sink);
  return hipGetLastError() == hipSuccess ? CB_OK : CB_EHIP;
}

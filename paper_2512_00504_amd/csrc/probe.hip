// Measurement aid: a plain streaming read of a device buffer with 128-bit loads, used by the
// benchmark to report the read bandwidth this GPU sustains next to the kernels' figures.
#include "gkv_internal.h"

namespace {

__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* sink) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint4 acc = make_uint4(0, 0, 0, 0);
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = src[i + k * stride];
#pragma unroll
    for (int k = 0; k < 8; ++k) { acc.x ^= v[k].x; acc.y ^= v[k].y; acc.z ^= v[k].z; acc.w ^= v[k].w; }
  }
  for (; i < n16; i += stride) { uint4 v = src[i]; acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
  // keeps the loads alive; the store itself practically never happens
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc.x;
}

}  // namespace

extern "C" gkv_status gkv_probe_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || bytes < 16) return GKV_ERR_INVALID_ARG;
  hipLaunchKernelGGL(stream_read_kernel, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream,
                     (const uint4*)src, bytes / 16, (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? GKV_OK : GKV_ERR_HIP;
}

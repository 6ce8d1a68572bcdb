// Measurement aid: the decode kernel's memory access pattern with no arithmetic, used by the
// benchmark to report the read rate the memory system grants that pattern next to the kernel's own.
#include "gkv_internal.h"
#include "gkv_bench.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Same slicing as attend_mfma_kernel: wavefront `wave` of the unit's workgroup takes the 16-row
// slices wave, wave+4, ...; per slice 4 loads of 1 KiB for the K tile (ordinary) and 4 loads of
// 4 x 256-byte V rows (non-temporal), the next slice issued right after the current one is consumed.
__global__ __launch_bounds__(256, 4) void attend_read_kernel(const char* __restrict__ K, const char* __restrict__ V,
                                                             int cap, int rows, uint32_t* sink) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, r = lane & 15, kb = lane >> 4;
  const char* Kh = K + (size_t)blockIdx.x * cap * 256;
  const char* Vh = V + (size_t)blockIdx.x * cap * 256;
  const int n_iter = rows >> 4;
  u32x4 acc = {0u, 0u, 0u, 0u};
  u32x4 cur[8];
  int it = wave;
  auto issue = [&](int i) {
    const char* Kt = Kh + (size_t)i * 4096;
#pragma unroll
    for (int c = 0; c < 4; ++c) cur[c] = *(const u32x4*)(Kt + c * 1024 + lane * 16);
#pragma unroll
    for (int jj = 0; jj < 4; ++jj)
      cur[4 + jj] = __builtin_nontemporal_load((const u32x4*)(Vh + (size_t)(16 * i + jj + 4 * kb) * 256 + r * 16));
  };
  if (it < n_iter) issue(it);
  while (it < n_iter) {
#pragma unroll
    for (int x = 0; x < 8; ++x) acc ^= cur[x];
    it += 4;
    if (it < n_iter) issue(it);
  }
  // keeps the loads alive; the store itself practically never happens
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) *sink = acc.x;
}

}  // namespace

extern "C" gkv_status gkv_probe_attend_read(const void* K, const void* V, int32_t units, int32_t capacity,
                                            int32_t rows, void* sink, void* stream) {
  if (!K || !V || !sink || units < 1 || capacity < 16 || rows < 16 || rows > capacity || (rows & 15))
    return GKV_ERR_INVALID_ARG;
  hipLaunchKernelGGL(attend_read_kernel, dim3(units), dim3(256), 0, (hipStream_t)stream,
                     (const char*)K, (const char*)V, (int)capacity, (int)rows, (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? GKV_OK : GKV_ERR_HIP;
}

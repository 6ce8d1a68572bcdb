// Internal declarations shared by the C-ABI layer and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gkv.h"
#include "gkv_bench.h"

// Dimensions every kernel needs, passed by value.
struct GkvDims {
  int32_t L, B, Hq, Hkv, d, g;
  int32_t b, w, s, cap;
  int32_t combine;
  float alpha;
  float scale;   // softmax scale of Eq. 1
  // scale * log2(e) as an unevaluated sum hi + lo: the matrix-core kernels form the exponent of
  // 2 as fma(z, lo, fma(z, hi, -m)), two roundings of a small number and no systematic error
  // from a rounded scale, and the decode and window-score kernels form it the same way
  float scale_l2_hi, scale_l2_lo;
  // Device-side step counter (null: none).  When set, the `step` argument of a call is relative
  // and the kernels use *step_base + step, so recorded launches (HIP graphs) can be replayed.
  const int32_t* step_base;
};

struct GkvProfile;   // event pools, defined in gkv_api.hip

struct gkv_ctx {
  gkv_config cfg;
  GkvDims dims;
  int32_t esz;            // bytes per element
  int32_t attend_splits;  // 0 = automatic
  int32_t ws_splits;      // split count the workspace was sized for by gkv_workspace_bytes (1 = no partials)
  int32_t attend_tile;    // keys per wavefront iteration of the matrix-core attend kernel: 16 or 32
  int32_t force_generic;
  int32_t attend_waves;   // 0 = automatic
  int32_t fuse_global;    // gkv_evict: global score in the tail of the window-score kernel
  int32_t fuse_select;    // gkv_evict: global score at the head of the top-k kernel (default)
  int32_t compact_ppt;    // 16-byte pieces per thread and chunk round of the compaction kernel: 4, 8 or 16
  int32_t reuse_stats;    // window score may reuse the softmax statistics the decode kernel recorded
  bool mfma_ok;           // bf16, d == 128, g <= 16
  GkvProfile* prof;
  // Host record of which ring slots hold softmax statistics written by the matrix-core decode
  // kernel: stats_step[slot] = decode step whose statistics the slot holds (-1 = none), valid for
  // exactly these buffers.
  int32_t* stats_step;    // [w]
  const void* stats_ws; const void* stats_K; const void* stats_qwin;
};

// Workspace layout (bytes from the base):
//   [0, 4*units)                    split tickets (int32, self-resetting)
//   [.., + 8*w*L*B*h_q)             softmax statistics ring: per (slot, layer, sequence, query head)
//                                   the running max (log2 units) and the sum of the decode step
//                                   whose q sits in that slot of the window ring
//   [.., + 4*units*splits*g*(d+2))  split-K partials (float)
struct GkvWorkspace {
  int32_t* split_ticket;
  int32_t* state_ticket;  // [L*B]: compaction workgroups of a (layer, sequence) that have finished; zero between launches
  float2* stats;
  float* partials;
};

static inline size_t gkv_align256(size_t x) { return (x + 255) & ~size_t(255); }

constexpr size_t GKV_LDS_LIMIT = 65536;
size_t gkv_max_lds_bytes(const gkv_config* cfg);
int gkv_effective_splits(const gkv_ctx* ctx);
GkvWorkspace gkv_carve_workspace(const gkv_ctx* ctx, void* base);

// Launch record for profiling: the wrappers launch through gkv_launch() below.
struct GkvLaunch {
  gkv_ctx* ctx;
  int kernel_id;
  hipStream_t stream;
};

// ---- launch wrappers implemented in the kernel files -------------------------------------
struct AttendArgs {
  const void* q; const void* k_new; const void* v_new;
  void* K; void* V; int32_t* pos; int32_t step; void* qwin; const int32_t* d_state; void* out;
  GkvWorkspace ws; int32_t splits; int32_t tile_keys;
  int32_t copy_q;   // 0 when q already is the ring slot of this step
  int32_t write_stats;   // record (max, sum) of every query head's softmax in ws.stats
  int32_t waves;         // wavefronts per workgroup of the matrix-core kernel: 4, 8 or 16
};
hipError_t gkv_launch_attend_generic(const GkvLaunch& ln, const GkvDims& dm, int dtype, const AttendArgs& a);
hipError_t gkv_launch_attend_mfma(const GkvLaunch& ln, const GkvDims& dm, const AttendArgs& a);

struct ScoreArgs {
  const void* qwin; const void* K; const int32_t* d_state; int32_t step; float* S;
  const float2* stats;   // softmax statistics of the window's decode steps, or null: compute them
  const float* F_hist; float* F_out;   // non-null F_out: also the global score (matrix-core kernel only)
};
hipError_t gkv_launch_score_generic(const GkvLaunch& ln, const GkvDims& dm, int dtype, const ScoreArgs& a);
hipError_t gkv_launch_score_mfma(const GkvLaunch& ln, const GkvDims& dm, const ScoreArgs& a);
bool gkv_score_mfma_supported(int g, int w, int cap);

hipError_t gkv_launch_global_update(const GkvLaunch& ln, const GkvDims& dm, const float* S,
                                    const float* F_hist, const int32_t* d_state, int32_t step, float* F_out);
hipError_t gkv_launch_select_topk(const GkvLaunch& ln, const GkvDims& dm, const float* F,
                                  const int32_t* d_state, int32_t step, int32_t* keep_idx);
hipError_t gkv_launch_update_and_select(const GkvLaunch& ln, const GkvDims& dm, const float* S, const float* F_hist,
                                        const int32_t* d_state, int32_t step, float* F_out, int32_t* keep_idx);
hipError_t gkv_launch_compact(const GkvLaunch& ln, const GkvDims& dm, int esz, const int32_t* keep_idx,
                              const float* F, void* K, void* V, float* F_hist, int32_t* pos,
                              int32_t* d_state, int32_t step, int32_t* state_ticket);
hipError_t gkv_launch_redundancy(const GkvLaunch& ln, const GkvDims& dm, int dtype, bool mfma, const void* K,
                                 const int32_t* d_state, int32_t step, const float* F, float lambda, float tau,
                                 float eps, int32_t n_recent, float* R_norm, float* F_sel);
hipError_t gkv_launch_pool_scores(const GkvLaunch& ln, const GkvDims& dm, const float* F, const int32_t* d_state,
                                  int32_t step, int32_t kernel, float* F_out);
hipError_t gkv_launch_evicted_positions(const GkvLaunch& ln, const GkvDims& dm, const int32_t* keep_idx,
                                        const int32_t* pos, const int32_t* d_state, int32_t step, int32_t* evicted);
hipError_t gkv_launch_fill_zero(hipStream_t stream, int32_t* p, size_t n);
hipError_t gkv_launch_add_int(hipStream_t stream, int32_t* p, int32_t delta);

// Event bracketing for profiling (gkv_api.hip).  Returns the events to pass to
// hipExtLaunchKernelGGL, or nulls when profiling is off.
void gkv_profile_events(const GkvLaunch& ln, hipEvent_t* start, hipEvent_t* stop);

// ---- device helpers ------------------------------------------------------------------------
#ifdef __HIPCC__
#include <hip/hip_ext.h>

template <typename... Args, typename F = void (*)(Args...)>
static inline hipError_t gkv_launch(const GkvLaunch& ln, F kernel, dim3 grid, dim3 block,
                                    size_t shmem, Args... args) {
  hipEvent_t e0 = nullptr, e1 = nullptr;
  gkv_profile_events(ln, &e0, &e1);
  if (e0) {
    hipExtLaunchKernelGGL(kernel, grid, block, shmem, ln.stream, e0, e1, 0, args...);
  } else {
    hipLaunchKernelGGL(kernel, grid, block, shmem, ln.stream, args...);
  }
  return hipGetLastError();
}

// The per-(layer, sequence) record of d_state, read with one 16-byte load.
struct SeqState {
  int32_t len, len_step, n_hist, n_tiled;
};
__device__ __forceinline__ SeqState load_state(const int32_t* d_state, int lb) {
  const int4 v = *(const int4*)(d_state + 4 * (size_t)lb);
  // the tiled prefix is whole tiles and never reaches past the stored length
  int nt = v.w & ~15;
  const int lim = (v.x > 0 ? v.x : 0) & ~15;
  nt = nt < 0 ? 0 : (nt > lim ? lim : nt);
  return SeqState{v.x, v.y, v.z, nt};
}
// Length before decode step `t` (every step since len_step appended one row), kept inside [0, cap].
__device__ __forceinline__ int length_before_step(const SeqState& s, int t, int cap) {
  const int l = s.len + (t - s.len_step);
  return l < 0 ? 0 : (l > cap ? cap : l);
}

// The decode step a kernel works on: its argument, plus the device-side step base if there is one.
__device__ __forceinline__ int resolve_step(const GkvDims& dm, int step) {
  return dm.step_base ? step + *dm.step_base : step;
}

// Whether the compression after decode step `step` applies to this (layer, sequence): its cache
// must exceed the budget, and the observation window must consist of generated tokens, i.e. at
// least w steps were decoded since the cache was loaded or last compacted (a prompt brings keys
// and values but no window queries).  Returns the length l the compression sees, or 0 for "skip".
__device__ __forceinline__ int compression_length(const SeqState& s, int step, int b, int w, int cap) {
  const int l = length_before_step(s, step + 1, cap);
  return (l > b && step + 1 - s.len_step >= w) ? l : 0;
}

// Element offset of (row n, channel c) in one KV head's K block whose first n_tiled rows are in
// tiled format; EPC = elements per 16 bytes.
template <int EPC>
__device__ __forceinline__ int k_elem_offset(int n, int c, int d, int n_tiled) {
  if (n >= n_tiled) return n * d + c;
  return (n >> 4) * 16 * d + (c / EPC) * (16 * EPC) + (n & 15) * EPC + (c % EPC);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) {
  return __uint_as_float(((uint32_t)b) << 16);
}
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {   // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int EPC = 4;
  __device__ static __forceinline__ float ld(const float* p) { return *p; }
  __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct Elem<uint16_t> {     // bf16 bit patterns
  static constexpr int EPC = 8;
  __device__ static __forceinline__ float ld(const uint16_t* p) { return bf16_bits_to_float(*p); }
  __device__ static __forceinline__ void st(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
// Block-wide reductions over blockDim.x = 256 threads; `red` is 8 floats of LDS.  The result is
// the same in every thread and independent of scheduling (fixed combination order).
__device__ __forceinline__ float block_max(float v, float* red) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r = fmaxf(r, red[i]);
  return r;
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = red[0];
  for (int i = 1; i < (int)(blockDim.x >> 6); ++i) r += red[i];
  return r;
}
#endif  // __HIPCC__

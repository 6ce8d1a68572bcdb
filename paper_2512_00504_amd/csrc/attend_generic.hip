// Decode attention, plain vector-ALU version for any dtype / head shape.
// One workgroup of 4 wavefronts per unit (layer, sequence, KV head); each wavefront takes the
// query heads hi = wave, wave + 4, ... of the group and does a whole head on its own (logits,
// softmax, output) with wavefront-level reductions only, so the heads of a group run side by
// side.  fp32 arithmetic throughout.  Used for the fp32 configuration and for shapes the
// matrix-core kernel does not cover.
#include "gkv_internal.h"

namespace {

constexpr int NWG = 4;     // wavefronts per workgroup

// Dynamic LDS, per wavefront: float prob[cap + 1]; float qs[d]
template <typename T>
__global__ __launch_bounds__(NWG * 64) void attend_generic_kernel(GkvDims dm, AttendArgs a) {
  a.step = resolve_step(dm, a.step);
  extern __shared__ float smem[];
  constexpr int EPC = Elem<T>::EPC;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int unit = blockIdx.x;
  const int j = unit % dm.Hkv;
  const int lb = unit / dm.Hkv;
  const int d = dm.d, cap = dm.cap, g = dm.g;
  float* prob = smem + (size_t)wave * (cap + 1 + d);
  float* qs = prob + cap + 1;

  const SeqState st = load_state(a.d_state, lb);
  const int len0 = length_before_step(st, a.step, cap);
  const bool has_new = (a.k_new != nullptr) && (len0 < cap);
  const int n_tot = len0 + (has_new ? 1 : 0);

  const T* Kh = (const T*)a.K + (size_t)unit * cap * d;
  const T* Vh = (const T*)a.V + (size_t)unit * cap * d;
  const T* kn = has_new ? (const T*)a.k_new + (size_t)unit * d : nullptr;
  const T* vn = has_new ? (const T*)a.v_new + (size_t)unit * d : nullptr;

  for (int hi = wave; hi < g; hi += NWG) {
    const int head = j * g + hi;
    const T* qh = (const T*)a.q + ((size_t)lb * dm.Hq + head) * d;
    for (int c = lane; c < d; c += 64) qs[c] = Elem<T>::ld(qh + c);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // logits: a lane per key
    float mx = -INFINITY;
    for (int n = lane; n < n_tot; n += 64) {
      float acc = 0.f;
      if (n == len0 && has_new) {
        for (int c = 0; c < d; ++c) acc = fmaf(qs[c], Elem<T>::ld(kn + c), acc);
      } else {
        for (int c = 0; c < d; ++c)
          acc = fmaf(qs[c], Elem<T>::ld(Kh + k_elem_offset<EPC>(n, c, d, st.n_tiled)), acc);
      }
      acc *= dm.scale;
      prob[n] = acc;
      mx = fmaxf(mx, acc);
    }
    mx = wave_max(mx);
    float sm = 0.f;
    for (int n = lane; n < n_tot; n += 64) {
      float e = expf(prob[n] - mx);
      prob[n] = e;
      sm += e;
    }
    sm = wave_sum(sm);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float inv = sm > 0.f ? 1.f / sm : 0.f;
    // output: a lane per channel, keys in order
    T* oh = (T*)a.out + ((size_t)lb * dm.Hq + head) * d;
    for (int c = lane; c < d; c += 64) {
      float acc = 0.f;
      for (int n = 0; n < len0; ++n) acc = fmaf(prob[n], Elem<T>::ld(Vh + (size_t)n * d + c), acc);
      if (has_new) acc = fmaf(prob[len0], Elem<T>::ld(vn + c), acc);
      Elem<T>::st(oh + c, acc * inv);
    }
    __builtin_amdgcn_wave_barrier();           // prob / qs are reused by this wavefront's next head
  }

  // Append the new row (row-major: len0 >= n_tiled always) and push q into the window ring,
  // after all reads of this unit's cache.
  __syncthreads();
  if (has_new) {
    T* Kw = (T*)a.K + (size_t)unit * cap * d;
    T* Vw = (T*)a.V + (size_t)unit * cap * d;
    for (int c = tid; c < d; c += blockDim.x) {
      Kw[(size_t)len0 * d + c] = kn[c];
      Vw[(size_t)len0 * d + c] = vn[c];
    }
    if (tid == 0) a.pos[(size_t)unit * cap + len0] = a.step;
  }
  if (a.copy_q) {
    const int slot = a.step % dm.w;
    const size_t nlb = (size_t)dm.L * dm.B;
    for (int x = tid; x < g * d; x += blockDim.x) {
      const int head = j * g + x / d, c = x % d;
      ((T*)a.qwin)[(((size_t)slot * nlb + lb) * dm.Hq + head) * d + c] =
          ((const T*)a.q)[((size_t)lb * dm.Hq + head) * d + c];
    }
  }
}

}  // namespace

hipError_t gkv_launch_attend_generic(const GkvLaunch& ln, const GkvDims& dm, int dtype, const AttendArgs& a) {
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(float) * NWG * (size_t)(dm.cap + 1 + dm.d);
  if (dtype == GKV_F32)
    return gkv_launch(ln, attend_generic_kernel<float>, dim3(units), dim3(NWG * 64), shmem, dm, a);
  return gkv_launch(ln, attend_generic_kernel<uint16_t>, dim3(units), dim3(NWG * 64), shmem, dm, a);
}

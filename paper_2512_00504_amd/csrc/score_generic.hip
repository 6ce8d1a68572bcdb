// Local score of the observation window, plain vector-ALU version (any dtype / shape).
// One workgroup per unit.  For each window row k and each query head of the group:
// softmax over the rows that query saw (Eq. 1), running max over the heads, then the
// mean over the window rows (Eq. 2).  Nothing but S leaves the chip.
#include "gkv_internal.h"

namespace {

// Dynamic LDS: float z[cap]; float rowmax[cap]; float sacc[cap]; float qs[d]; float red[8]
template <typename T>
__global__ __launch_bounds__(256) void score_generic_kernel(GkvDims dm, ScoreArgs a) {
  extern __shared__ float smem[];
  constexpr int EPC = Elem<T>::EPC;
  const int tid = threadIdx.x;
  const int unit = blockIdx.x;
  const int j = unit % dm.Hkv;
  const int lb = unit / dm.Hkv;
  const int d = dm.d, cap = dm.cap, g = dm.g, w = dm.w;
  float* z = smem;
  float* rowmax = z + cap;
  float* sacc = rowmax + cap;
  float* qs = sacc + cap;
  float* red = qs + d;

  const SeqState st = load_state(a.d_state, lb);
  const int l = length_before_step(st, a.step + 1, cap);
  if (l <= dm.b) return;                     // not above the budget: no compression for this sequence
  const int c = l - w;
  const T* Kh = (const T*)a.K + (size_t)unit * cap * d;

  for (int n = tid; n < c; n += blockDim.x) sacc[n] = 0.f;
  for (int k = 0; k < w; ++k) {
    const int t_row = a.step - w + 1 + k;                 // decode step of window row k
    const int slot = ((t_row % w) + w) % w;
    const int n_vis = c + k + 1;                          // rows [0, c+k] were visible to it
    for (int n = tid; n < c; n += blockDim.x) rowmax[n] = 0.f;
    for (int hi = 0; hi < g; ++hi) {
      const int head = j * g + hi;
      const T* qh = (const T*)a.qwin + (((size_t)slot * dm.L * dm.B + lb) * dm.Hq + head) * d;
      __syncthreads();
      for (int ch = tid; ch < d; ch += blockDim.x) qs[ch] = Elem<T>::ld(qh + ch);
      __syncthreads();
      float mx = -INFINITY;
      for (int n = tid; n < n_vis; n += blockDim.x) {
        float acc = 0.f;
        for (int ch = 0; ch < d; ++ch) acc = fmaf(qs[ch], Elem<T>::ld(Kh + k_elem_offset<EPC>(n, ch, d, st.n_tiled)), acc);
        acc *= dm.scale;
        z[n] = acc;
        mx = fmaxf(mx, acc);
      }
      mx = block_max(mx, red);
      float sm = 0.f;
      for (int n = tid; n < n_vis; n += blockDim.x) {
        float e = expf(z[n] - mx);
        z[n] = e;
        sm += e;
      }
      sm = block_sum(sm, red);
      for (int n = tid; n < c; n += blockDim.x) rowmax[n] = fmaxf(rowmax[n], z[n] / sm);
    }
    for (int n = tid; n < c; n += blockDim.x) sacc[n] += rowmax[n];
  }
  float* So = a.S + (size_t)unit * cap;
  for (int n = tid; n < c; n += blockDim.x) So[n] = sacc[n] / (float)w;
}

}  // namespace

hipError_t gkv_launch_score_generic(const GkvLaunch& ln, const GkvDims& dm, int dtype, const ScoreArgs& a) {
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(float) * (3 * (size_t)dm.cap + dm.d + 8);
  if (dtype == GKV_F32)
    return gkv_launch(ln, score_generic_kernel<float>, dim3(units), dim3(256), shmem, dm, a);
  return gkv_launch(ln, score_generic_kernel<uint16_t>, dim3(units), dim3(256), shmem, dm, a);
}

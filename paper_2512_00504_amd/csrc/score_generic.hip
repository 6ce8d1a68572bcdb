// Local score of the observation window, plain vector-ALU version (any dtype / shape).
// One workgroup per unit; each wavefront takes window rows k = wave, wave + nw, ... and for
// each does, head by head: softmax over the rows that query saw (Eq. 1), running max over the
// heads of the group, then adds the row into its partial sum over the window (Eq. 2).  The
// wavefronts' partial sums are added in wavefront order.  Nothing but S leaves the chip.
#include "gkv_internal.h"

namespace {

// Dynamic LDS, per wavefront: float z[cap]; float rowmax[cap]; float sacc[cap]; float qs[d]
template <typename T>
__global__ void score_generic_kernel(GkvDims dm, ScoreArgs a) {
  a.step = resolve_step(dm, a.step);
  extern __shared__ float smem[];
  constexpr int EPC = Elem<T>::EPC;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  const int unit = blockIdx.x;
  const int j = unit % dm.Hkv;
  const int lb = unit / dm.Hkv;
  const int d = dm.d, cap = dm.cap, g = dm.g, w = dm.w;
  const size_t per_wave = 3 * (size_t)cap + d;
  float* z = smem + wave * per_wave;
  float* rowmax = z + cap;
  float* sacc = rowmax + cap;
  float* qs = sacc + cap;

  const SeqState st = load_state(a.d_state, lb);
  const int l = compression_length(st, a.step, dm.b, w, cap);
  if (l == 0) return;                        // at or below the budget, or window not full: no compression
  const int c = l - w;
  const T* Kh = (const T*)a.K + (size_t)unit * cap * d;

  for (int n = lane; n < c; n += 64) sacc[n] = 0.f;
  for (int k = wave; k < w; k += nw) {
    const int t_row = a.step - w + 1 + k;                 // decode step of window row k
    const int slot = ((t_row % w) + w) % w;
    const int n_vis = c + k + 1;                          // rows [0, c+k] were visible to it
    for (int n = lane; n < c; n += 64) rowmax[n] = 0.f;
    for (int hi = 0; hi < g; ++hi) {
      const int head = j * g + hi;
      const T* qh = (const T*)a.qwin + (((size_t)slot * dm.L * dm.B + lb) * dm.Hq + head) * d;
      __builtin_amdgcn_wave_barrier();
      for (int ch = lane; ch < d; ch += 64) qs[ch] = Elem<T>::ld(qh + ch);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      float mx = -INFINITY;
      for (int n = lane; n < n_vis; n += 64) {
        float acc = 0.f;
        for (int ch = 0; ch < d; ++ch)
          acc = fmaf(qs[ch], Elem<T>::ld(Kh + k_elem_offset<EPC>(n, ch, d, st.n_tiled)), acc);
        acc *= dm.scale;
        z[n] = acc;
        mx = fmaxf(mx, acc);
      }
      mx = wave_max(mx);
      float sm = 0.f;
      for (int n = lane; n < n_vis; n += 64) {
        float e = expf(z[n] - mx);
        z[n] = e;
        sm += e;
      }
      sm = wave_sum(sm);
      for (int n = lane; n < c; n += 64) rowmax[n] = fmaxf(rowmax[n], z[n] / sm);   // each lane its own n
    }
    for (int n = lane; n < c; n += 64) sacc[n] += rowmax[n];
  }
  __syncthreads();
  float* So = a.S + (size_t)unit * cap;
  for (int n = tid; n < c; n += blockDim.x) {
    float tot = 0.f;
    for (int wv = 0; wv < nw; ++wv) tot += smem[wv * per_wave + 2 * (size_t)cap + n];
    So[n] = tot / (float)w;
  }
}

}  // namespace

hipError_t gkv_launch_score_generic(const GkvLaunch& ln, const GkvDims& dm, int dtype, const ScoreArgs& a) {
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t per_wave = sizeof(float) * (3 * (size_t)dm.cap + dm.d);
  int nw = (int)(65536 / per_wave);
  nw = nw < 1 ? 1 : (nw > 4 ? 4 : nw);
  const size_t shmem = per_wave * nw;
  if (dtype == GKV_F32)
    return gkv_launch(ln, score_generic_kernel<float>, dim3(units), dim3(nw * 64), shmem, dm, a);
  return gkv_launch(ln, score_generic_kernel<uint16_t>, dim3(units), dim3(nw * 64), shmem, dm, a);
}

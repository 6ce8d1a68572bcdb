// Decode attention on the matrix cores: bf16, head_dim 128, group size g <= 16.
//
// One workgroup of NW wavefronts per (unit, split).  A wavefront owns 32-key slices of the
// cache (slice it, it + splits*NW, ...) and keeps flash-decoding state (running max, running
// sum, fp32 accumulators) for all g query heads of the KV group, so K and V are read from
// HBM exactly once per KV head.
//
// Per 32-key slice and wavefront:
//   K: two 16-key tiles.  The tiled K layout makes each matrix-core A operand
//      (16 keys x 32 channels, lane = key + 16*kblock) one contiguous 1 KiB load.
//      S^T[key, head] = K[key, :] . Q[head, :]  -> 4 MFMA 16x16x32 per tile.
//      The result lane (head = lane%16, blk = lane/16) holds 8 keys of its head.
//   softmax: running max shared by the 4 lanes of a head (2 cross-lane exchanges), exp2.
//   V: lane (chunk = lane%16, kb = lane/16) loads the 16-byte chunk `chunk` of 8 keys, so a
//      quarter-wave reads one full 256-byte row per load.  An 8x8 in-register transpose
//      (v_perm_b32) turns that into A operands V^T[channel, key]; with B = P^T[key, head]
//      (the probabilities, already in the right lanes) 8 MFMAs give O^T[channel, head].
// The wavefronts of a workgroup are merged through LDS; splits of one unit are merged by the
// last workgroup to finish (ticket counter), in a fixed order, so results are deterministic.
//
// The newest token's k/v are not read from the cache (another workgroup may be writing that
// row): the lanes that would hold row `len` take them from k_new / v_new instead.
#include "gkv_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int ROW_BYTES = D * 2;          // 256
constexpr int TILE_BYTES = 16 * ROW_BYTES;
constexpr int OSTR = D + 4;               // padded LDS row of the per-wave partial outputs
constexpr int PSTR = D + 2;               // split-K partial: o[128], m, l

__device__ __forceinline__ u32x4 ld16(const void* p) { return *(const u32x4*)p; }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

template <int NW>
__global__ __launch_bounds__(NW * 64) void attend_mfma_kernel(GkvDims dm, AttendArgs a) {
  extern __shared__ float smem[];
  __shared__ int s_misc[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kb = lane >> 4;
  const int splits = a.splits;
  const int unit = blockIdx.x / splits, sp = blockIdx.x % splits;
  const int j = unit % dm.Hkv, lb = unit / dm.Hkv;
  const int g = dm.g, cap = dm.cap;

  if (tid == 0) s_misc[0] = a.d_len[lb];
  __syncthreads();
  const int len0 = s_misc[0];
  const bool has_new = (a.k_new != nullptr) && (len0 < cap);
  if (tid == 0) {
    // ticket: the last workgroup of this (layer, sequence) to have read the length bumps it
    int old = atomicAdd(&a.ws.len_ticket[lb], 1);
    if (old == dm.Hkv * splits - 1) {
      a.ws.len_ticket[lb] = 0;
      if (has_new) a.d_len[lb] = len0 + 1;
    }
  }
  const int n_tot = len0 + (has_new ? 1 : 0);

  const char* Kh = (const char*)a.K + (size_t)unit * cap * ROW_BYTES;
  const char* Vh = (const char*)a.V + (size_t)unit * cap * ROW_BYTES;
  const char* knew = (const char*)a.k_new + (size_t)unit * ROW_BYTES;
  const char* vnew = (const char*)a.v_new + (size_t)unit * ROW_BYTES;

  // B operand of the QK product: lane (head r, kblock kb) holds channels [8*(4c+kb), +8) of q[r]
  bf16x8 qB[4];
  {
    const char* qh = (const char*)a.q + ((size_t)lb * dm.Hq + j * g + r) * ROW_BYTES;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < g) v = ld16(qh + (4 * c + kb) * 16);
      qB[c] = as_bf16x8(v);
    }
  }
  const float scale_log2 = dm.scale * 1.4426950408889634f;

  float m_run = -1e30f, l_run = 0.f;
  f32x4 oacc[8];
#pragma unroll
  for (int m = 0; m < 8; ++m) oacc[m] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int n_iter = (n_tot + 31) >> 5;
  for (int it = sp * NW + wave; it < n_iter; it += splits * NW) {
    const int key0 = it << 5;
    const char* Kt = Kh + (size_t)(key0 >> 4) * TILE_BYTES;
    u32x4 kA[2][4];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt)
#pragma unroll
      for (int c = 0; c < 4; ++c) kA[tt][c] = ld16(Kt + tt * TILE_BYTES + c * 1024 + lane * 16);
    u32x4 vR[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
      vR[jj] = ld16(Vh + (size_t)key * ROW_BYTES + r * 16);
    }
    if (has_new && key0 <= len0 && len0 < key0 + 32) {       // wave-uniform
      const int tt_new = (len0 - key0) >> 4, rr = len0 & 15;
#pragma unroll
      for (int tt = 0; tt < 2; ++tt)
        if (tt == tt_new && r == rr) {
#pragma unroll
          for (int c = 0; c < 4; ++c) kA[tt][c] = ld16(knew + (4 * c + kb) * 16);
        }
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
        if (key == len0) vR[jj] = ld16(vnew + r * 16);
      }
    }
    const bool tail = key0 + 32 > n_tot;                        // wave-uniform
    if (tail) {
#pragma unroll
      for (int jj = 0; jj < 8; ++jj) {
        const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
        if (key >= n_tot) vR[jj] = u32x4{0u, 0u, 0u, 0u};    // stale rows must not reach the MFMA
      }
    }

    // scores: sc[tt][e] = q[head r] . k[key0 + 16 tt + 4 kb + e]
    f32x4 sc[2];
#pragma unroll
    for (int tt = 0; tt < 2; ++tt) {
      sc[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < 4; ++c)
        sc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[tt][c]), qB[c], sc[tt], 0, 0, 0);
    }
    float s8[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      s8[i] = sc[i >> 2][i & 3] * scale_log2;
      if (tail) {
        const int key = key0 + (i >> 2) * 16 + 4 * kb + (i & 3);
        if (key >= n_tot) s8[i] = -INFINITY;
      }
    }
    float mx = s8[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) mx = fmaxf(mx, s8[i]);
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    if (__any(m_new > m_run)) {
      const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
      l_run *= corr;
#pragma unroll
      for (int m = 0; m < 8; ++m) oacc[m] *= corr;
      m_run = m_new;
    }
    f32x8 p8;
    float psum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p = __builtin_amdgcn_exp2f(s8[i] - m_run);
      p8[i] = p;
      psum += p;
    }
    l_run += psum;
    const bf16x8 pB = __builtin_convertvector(p8, bf16x8);

    // O^T[channel 8*(4 blk + e) + m, head] += V^T . P^T
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      u32x4 t;
#pragma unroll
      for (int y = 0; y < 4; ++y)
        t[y] = __builtin_amdgcn_perm(vR[2 * y + 1][m >> 1], vR[2 * y][m >> 1],
                                     (m & 1) ? 0x07060302u : 0x05040100u);
      oacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t), pB, oacc[m], 0, 0, 0);
    }
  }

  // ---- merge the wavefronts of this workgroup -------------------------------------------------
  float* so = smem;                         // [NW][g][OSTR]
  float* sm = so + NW * g * OSTR;           // [NW][16]
  float* sl = sm + NW * 16;                 // [NW][4][16]
  if (r < g) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float* dst = so + (wave * g + r) * OSTR + 32 * kb + 8 * e;
      *(f32x4*)dst = f32x4{oacc[0][e], oacc[1][e], oacc[2][e], oacc[3][e]};
      *(f32x4*)(dst + 4) = f32x4{oacc[4][e], oacc[5][e], oacc[6][e], oacc[7][e]};
    }
    sl[(wave * 4 + kb) * 16 + r] = l_run;
    if (kb == 0) sm[wave * 16 + r] = m_run;
  }
  __syncthreads();

  uint16_t* out = (uint16_t*)a.out + ((size_t)lb * dm.Hq + j * g) * D;
  float* part = a.ws.partials + (size_t)(unit * splits + sp) * g * PSTR;
  for (int x = tid; x < g * 64; x += NW * 64) {
    const int h = x >> 6, cp = x & 63;
    float M = sm[h];
#pragma unroll
    for (int wv = 1; wv < NW; ++wv) M = fmaxf(M, sm[wv * 16 + h]);
    float Lsum = 0.f, o0 = 0.f, o1 = 0.f;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const float f = __builtin_amdgcn_exp2f(sm[wv * 16 + h] - M);
      const float lw = (sl[(wv * 4 + 0) * 16 + h] + sl[(wv * 4 + 1) * 16 + h]) +
                       (sl[(wv * 4 + 2) * 16 + h] + sl[(wv * 4 + 3) * 16 + h]);
      Lsum += lw * f;
      o0 += so[(wv * g + h) * OSTR + 2 * cp] * f;
      o1 += so[(wv * g + h) * OSTR + 2 * cp + 1] * f;
    }
    if (splits == 1) {
      const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
      const uint32_t packed = (uint32_t)float_to_bf16_bits(o0 * inv) |
                              ((uint32_t)float_to_bf16_bits(o1 * inv) << 16);
      *(uint32_t*)(out + h * D + 2 * cp) = packed;
    } else {
      float* ph = part + h * PSTR;
      ph[2 * cp] = o0;
      ph[2 * cp + 1] = o1;
      if (cp == 0) { ph[D] = M; ph[D + 1] = Lsum; }
    }
  }

  // ---- merge the splits of this unit: last workgroup to finish does it ------------------------
  if (splits > 1) {
    __threadfence();
    __syncthreads();
    if (tid == 0) {
      const int old = atomicAdd(&a.ws.split_ticket[unit], 1);
      s_misc[1] = (old == splits - 1);
      if (old == splits - 1) a.ws.split_ticket[unit] = 0;
    }
    __syncthreads();
    if (s_misc[1]) {
      __threadfence();
      const float* pu = a.ws.partials + (size_t)unit * splits * g * PSTR;
      for (int x = tid; x < g * 64; x += NW * 64) {
        const int h = x >> 6, cp = x & 63;
        float M = -1e30f;
        for (int s2 = 0; s2 < splits; ++s2) M = fmaxf(M, pu[(s2 * g + h) * PSTR + D]);
        float Lsum = 0.f, o0 = 0.f, o1 = 0.f;
        for (int s2 = 0; s2 < splits; ++s2) {
          const float* ph = pu + (s2 * g + h) * PSTR;
          const float f = __builtin_amdgcn_exp2f(ph[D] - M);
          Lsum += ph[D + 1] * f;
          o0 += ph[2 * cp] * f;
          o1 += ph[2 * cp + 1] * f;
        }
        const float inv = Lsum > 0.f ? 1.f / Lsum : 0.f;
        const uint32_t packed = (uint32_t)float_to_bf16_bits(o0 * inv) |
                                ((uint32_t)float_to_bf16_bits(o1 * inv) << 16);
        *(uint32_t*)(out + h * D + 2 * cp) = packed;
      }
    }
  }

  // ---- append the new row, push q into the window ring (split 0 only) -------------------------
  if (sp == 0) {
    if (has_new) {
      if (tid < 16) {
        *(u32x4*)((char*)a.K + (size_t)unit * cap * ROW_BYTES + (size_t)(len0 >> 4) * TILE_BYTES +
                  tid * 256 + (len0 & 15) * 16) = ld16(knew + tid * 16);
      } else if (tid < 32) {
        const int ch = tid - 16;
        *(u32x4*)((char*)a.V + (size_t)unit * cap * ROW_BYTES + (size_t)len0 * ROW_BYTES + ch * 16) =
            ld16(vnew + ch * 16);
      } else if (tid == 32) {
        a.pos[(size_t)unit * cap + len0] = a.step;
      }
    }
    const int slot = a.step % dm.w;
    for (int x = tid; x < g * 16; x += NW * 64) {
      const int h = x >> 4, ch = x & 15;
      const size_t head = (size_t)lb * dm.Hq + j * g + h;
      *(u32x4*)((char*)a.qwin + ((head * dm.w + slot) * (size_t)ROW_BYTES) + ch * 16) =
          ld16((const char*)a.q + head * ROW_BYTES + ch * 16);
    }
  }
}

}  // namespace

hipError_t gkv_launch_attend_mfma(const GkvLaunch& ln, const GkvDims& dm, const AttendArgs& a) {
  constexpr int NW = 4;
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(float) * (NW * dm.g * OSTR + NW * 16 + NW * 64);
  return gkv_launch(ln, attend_mfma_kernel<NW>, dim3(units * a.splits), dim3(NW * 64), shmem, dm, a);
}

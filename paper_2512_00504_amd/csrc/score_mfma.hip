// Local score of the observation window on the matrix cores: bf16, head_dim 128,
// w a multiple of 16, group sizes instantiated below.
//
// One workgroup (NW wavefronts) per unit.  The window queries of the group's G heads are
// staged in LDS once, in window-row order.  A wavefront takes 16-key tiles of K (one 1 KiB
// contiguous load per 32 channels, thanks to the tiled K layout) and for every (head, block
// of 16 window rows) computes logits^T[key, row] with 4 MFMA 16x16x32.
//   row statistics (max, sum of exponentials) of Eq. 1 over the keys each window row saw: under
//           the causal reading these are what the decode kernel computed when the row's query was
//           decoded, and it records them next to the window ring; they are taken from there, or,
//           when the last w decode calls were not this window's, computed by a first pass over K;
//   scores: logits of the candidates, p = 2^(z*scale*log2e - max)/sum, running max over the
//           heads in registers (group max-reduce), then the sum over the 16 lanes that hold the
//           window rows (Eq. 2).  Only S leaves the chip; the [g, w, l] matrix never exists in memory.
#include "gkv_internal.h"

#ifndef GKV_SCORE_NW
#define GKV_SCORE_NW 8      // wavefronts per workgroup
#endif

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int ROW_BYTES = D * 2;
constexpr int TILE_BYTES = 16 * ROW_BYTES;
constexpr int QSTR = ROW_BYTES + 16;       // padded LDS row of a staged query (bank spread)

__device__ __forceinline__ u32x4 ld16(const void* p) { return *(const u32x4*)p; }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// Probabilities are 2^(z*(hi+lo) - m) / sum with hi + lo = scale * log2(e) as an unevaluated sum
// and the exponent formed as fma(z, lo, fma(z, hi, -m)): the result of each fma is a small
// number (the distance from the row maximum in log2 units), so its rounding costs ~1e-7
// relative in the probability, and the rounding of the scale itself, which would act like a
// slightly different softmax temperature, is carried by lo.  The hardware exp2 is good to 1 ulp.
// The decode kernel forms its exponents the same way from bit-identical logits (same matrix-core
// instruction sequence over the same operands), which is what makes its recorded (max, sum) the
// row statistics of this kernel.
__device__ __forceinline__ float exp2_of(float z, float m, float hi, float lo) {
  return __builtin_amdgcn_exp2f(fmaf(z, lo, fmaf(z, hi, -m)));
}

// A operand of tile T: lane (row r, kblock kb) gets chunk 4c+kb of key 16T+r for c = 0..3; tiled
// tiles are lane-contiguous, row-major tiles (rows appended since the last compaction) are not.
// Sum over the 16 lanes of a DPP row (lanes 16i .. 16i+15), left in every one of them: lanes ^1
// and ^2 of each quad, then the other quad of each 8 (mirror within 8: the four lanes of a quad
// are equal by then), then the other 8 (mirror within 16).  Same pairs, same order as a butterfly
// over lane ^1, ^2, ^4, ^8, so the same bits, without four dependent trips through LDS.
__device__ __forceinline__ float row16_sum(float v) {
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false));   // row_half_mirror
  v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, false));   // row_mirror
  return v;
}

__device__ __forceinline__ void load_k_tile(u32x4 (&kA)[4], const char* Kh, int T, int n_tiled,
                                            int lane, int r, int kb) {
  const bool tiled = 16 * T < n_tiled;
  const char* p = Kh + (size_t)T * TILE_BYTES + (tiled ? lane * 16 : r * ROW_BYTES + kb * 16);
  const int step_off = tiled ? 1024 : 64;
#pragma unroll
  for (int c = 0; c < 4; ++c) kA[c] = ld16(p + c * step_off);
}

// Dynamic LDS: char qs[G*w*QSTR]; float rowM[G*w]; float rowZ[G*w]; float sbuf[cap]; float red[8]; and,
// when the row statistics are computed here, float redM[NW*G*w]; float redS[NW*G*w]
// HAVE_STATS: a.stats holds (max, sum) of every window row, recorded by the decode kernel.
template <int NW, int G, int WT, bool HAVE_STATS>
__global__ __launch_bounds__(NW * 64) void score_mfma_kernel(GkvDims dm, ScoreArgs a) {
  a.step = resolve_step(dm, a.step);
  extern __shared__ __attribute__((aligned(16))) char smem_raw[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kb = lane >> 4;
  const int unit = blockIdx.x, j = unit % dm.Hkv, lb = unit / dm.Hkv;
  const int cap = dm.cap;
  constexpr int W = 16 * WT;
  constexpr int ROWS = G * W;

  const SeqState seq = load_state(a.d_state, lb);
  const int l = compression_length(seq, a.step, dm.b, W, cap);
  if (l == 0) return;
  const int cc = l - W;                     // number of candidates

  char* qs = smem_raw;
  float* rowM = (float*)(qs + ROWS * QSTR);
  float* rowZ = rowM + ROWS;
  float* sbuf = rowZ + ROWS;                // S of this unit, for the fused global-score tail
  float* red = sbuf + cap;

  // stage the window queries: LDS row h*W + k holds head h, window row k (k-th oldest)
  for (int x = tid; x < ROWS * 16; x += NW * 64) {
    const int row = x >> 4, ch = x & 15;
    const int h = row / W, k = row % W;
    const int t_row = a.step - W + 1 + k;
    const int slot = ((t_row % W) + W) % W;
    *(u32x4*)(qs + row * QSTR + ch * 16) =
        ld16((const char*)a.qwin + (((size_t)slot * dm.L * dm.B + lb) * dm.Hq + j * G + h) * (size_t)ROW_BYTES + ch * 16);
  }
  if constexpr (HAVE_STATS) {
    for (int x = tid; x < ROWS; x += NW * 64) {
      const int h = x / W, k = x % W;
      const int t_row = a.step - W + 1 + k;
      const int slot = ((t_row % W) + W) % W;
      const float2 ms = a.stats[((size_t)slot * dm.L * dm.B + lb) * dm.Hq + j * G + h];
      rowM[x] = ms.x;
      rowZ[x] = 1.f / ms.y;
    }
  }
  __syncthreads();

  const char* Kh = (const char*)a.K + (size_t)unit * cap * ROW_BYTES;
  const float s_hi = dm.scale_l2_hi, s_lo = dm.scale_l2_lo;
  float rm[G][WT], rs[G][WT];

  if constexpr (!HAVE_STATS) {
    // ---- pass 1: row max and row sum over the keys visible to each window row -----------------
    // Only the last tiles (those reaching into the window) need the causal mask; the running sum
    // is rescaled only when some lane's maximum moved.
    float* redM = red + 8;
    float* redS = redM + NW * ROWS;
    const int n_tiles = (l + 15) >> 4;
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int nt = 0; nt < WT; ++nt) { rm[h][nt] = -1e30f; rs[h][nt] = 0.f; }

    for (int T = wave; T < n_tiles; T += NW) {
      u32x4 kA[4];
      load_k_tile(kA, Kh, T, seq.n_tiled, lane, r, kb);
      const int key_base = 16 * T + 4 * kb;
      const bool full = 16 * T + 15 <= cc;                    // every row sees all 16 keys of this tile
#pragma unroll
      for (int h = 0; h < G; ++h)
#pragma unroll
        for (int nt = 0; nt < WT; ++nt) {
          const char* qrow = qs + (h * W + 16 * nt + r) * QSTR;
          f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int c = 0; c < 4; ++c)
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[c]),
                                                          as_bf16x8(*(const u32x4*)(qrow + (4 * c + kb) * 16)),
                                                          acc, 0, 0, 0);
          float z[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) z[e] = acc[e];
          if (!full) {
            const int last_vis = cc + 16 * nt + r;            // row k sees keys [0, cc + k]
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (key_base + e > last_vis) z[e] = -1e30f;
          }
          const float tm = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3])) * s_hi;
          if (__any(tm > rm[h][nt])) {
            const float mnew = fmaxf(rm[h][nt], tm);
            rs[h][nt] *= __builtin_amdgcn_exp2f(rm[h][nt] - mnew);
            rm[h][nt] = mnew;
          }
          rs[h][nt] += (exp2_of(z[0], rm[h][nt], s_hi, s_lo) + exp2_of(z[1], rm[h][nt], s_hi, s_lo)) +
                       (exp2_of(z[2], rm[h][nt], s_hi, s_lo) + exp2_of(z[3], rm[h][nt], s_hi, s_lo));
        }
    }
    // merge the 4 lanes of a row, then the wavefronts
#pragma unroll
    for (int h = 0; h < G; ++h)
#pragma unroll
      for (int nt = 0; nt < WT; ++nt) {
        float m = rm[h][nt];
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        float s = rs[h][nt] * __builtin_amdgcn_exp2f(rm[h][nt] - m);
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (kb == 0) {
          redM[wave * ROWS + h * W + 16 * nt + r] = m;
          redS[wave * ROWS + h * W + 16 * nt + r] = s;
        }
      }
    __syncthreads();
    for (int x = tid; x < ROWS; x += NW * 64) {
      float M = redM[x];
#pragma unroll
      for (int wv = 1; wv < NW; ++wv) M = fmaxf(M, redM[wv * ROWS + x]);
      float Z = 0.f;
#pragma unroll
      for (int wv = 0; wv < NW; ++wv) Z += redS[wv * ROWS + x] * __builtin_amdgcn_exp2f(redM[wv * ROWS + x] - M);
      rowM[x] = M;
      rowZ[x] = 1.f / Z;                                       // one division per row, not per logit
    }
    __syncthreads();
  }
#pragma unroll
  for (int h = 0; h < G; ++h)
#pragma unroll
    for (int nt = 0; nt < WT; ++nt) {
      rm[h][nt] = rowM[h * W + 16 * nt + r];
      rs[h][nt] = rowZ[h * W + 16 * nt + r];
    }

  // ---- probabilities of the candidates, max over heads, mean over window rows ---------------
  float* So = a.S + (size_t)unit * cap;
  const int cand_tiles = (cc + 15) >> 4;
  const float wf = (float)W;
  u32x4 kA[4], kN[4];
  if (wave < cand_tiles) load_k_tile(kA, Kh, wave, seq.n_tiled, lane, r, kb);
  for (int T = wave; T < cand_tiles; T += NW) {
    // the wavefront's next tile is requested before this one is worked on (clamped at the end:
    // the same number of requests in flight on every path keeps the wait for this tile short)
    load_k_tile(kN, Kh, min(T + NW, cand_tiles - 1), seq.n_tiled, lane, r, kb);
    f32x4 tot = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int nt = 0; nt < WT; ++nt) {
      f32x4 amax = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int h = 0; h < G; ++h) {
        const char* qrow = qs + (h * W + 16 * nt + r) * QSTR;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[c]),
                                                        as_bf16x8(*(const u32x4*)(qrow + (4 * c + kb) * 16)),
                                                        acc, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // candidates are visible to every window row; keys >= cc are discarded below
          const float p = exp2_of(acc[e], rm[h][nt], s_hi, s_lo) * rs[h][nt];
          amax[e] = fmaxf(amax[e], p);
        }
      }
      tot += amax;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float v = row16_sum(tot[e]);
      const int key = 16 * T + 4 * kb + e;
      if (r == 0 && key < cc) { const float sv = v / wf; So[key] = sv; sbuf[key] = sv; }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) kA[c] = kN[c];
  }

  // ---- optional tail: global score of the candidates (Section 4), S still in LDS ---------------
  if (a.F_out != nullptr) {
    __syncthreads();
    float mx = 0.f;
    for (int n = tid; n < cc; n += NW * 64) mx = fmaxf(mx, sbuf[n]);
    mx = block_max(mx, red);
    const int n_hist = seq.n_hist < 0 ? 0 : (seq.n_hist > cc ? cc : seq.n_hist);
    const float* Hu = a.F_hist + (size_t)unit * cap;
    float* Fu = a.F_out + (size_t)unit * cap;
    for (int n = tid; n < cc; n += NW * 64) {
      const float sn = mx > 0.f ? sbuf[n] / mx : 0.f;
      float f = sn;
      if (n < n_hist) {
        const float h = dm.alpha * Hu[n];
        f = dm.combine == GKV_COMBINE_MAX ? fmaxf(h, sn)
          : dm.combine == GKV_COMBINE_AVG ? h + (1.f - dm.alpha) * sn
                                          : h + sn;
      }
      Fu[n] = f;
    }
  }
}

template <int G, int WT>
hipError_t launch(const GkvLaunch& ln, const GkvDims& dm, const ScoreArgs& a) {
  constexpr int NW = GKV_SCORE_NW;
  constexpr int ROWS = G * 16 * WT;
  const int units = dm.L * dm.B * dm.Hkv;
  if (a.stats) {
    const size_t shmem = (size_t)ROWS * QSTR + sizeof(float) * (2 * ROWS + dm.cap + 8);
    return gkv_launch(ln, score_mfma_kernel<NW, G, WT, true>, dim3(units), dim3(NW * 64), shmem, dm, a);
  }
  const size_t shmem = (size_t)ROWS * QSTR + sizeof(float) * (2 * ROWS + dm.cap + 8 + 2 * NW * ROWS);
  return gkv_launch(ln, score_mfma_kernel<NW, G, WT, false>, dim3(units), dim3(NW * 64), shmem, dm, a);
}

}  // namespace

bool gkv_score_mfma_supported(int g, int w, int cap) {
  const bool g_ok = (g == 1 || g == 2 || g == 4 || g == 5 || g == 7 || g == 8);
  if (!g_ok || (w != 16 && w != 32)) return false;
  const size_t rows = (size_t)g * w;                      // LDS the kernel needs; 64 KiB available
  return rows * QSTR + sizeof(float) * (2 * rows + 2 * GKV_SCORE_NW * rows + cap + 8) <= 65536;
}

hipError_t gkv_launch_score_mfma(const GkvLaunch& ln, const GkvDims& dm, const ScoreArgs& a) {
  const int wt = dm.w / 16;
#define GKV_CASE(G_)                                                        \
  if (dm.g == G_) return wt == 1 ? launch<G_, 1>(ln, dm, a) : launch<G_, 2>(ln, dm, a);
  GKV_CASE(1) GKV_CASE(2) GKV_CASE(4) GKV_CASE(5) GKV_CASE(7) GKV_CASE(8)
#undef GKV_CASE
  return hipErrorInvalidValue;
}

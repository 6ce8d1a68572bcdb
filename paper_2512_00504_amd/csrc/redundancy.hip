// Redundancy score of the cached keys and its combination with the global score
// (paper, appendix "Integrating the Global Score with Other Methods"):
//   Kn = K / (||K|| + eps);  C = Kn Kn^T;  entries below tau, the diagonal and the columns of
//   the n_recent newest rows are zeroed;  col_j = sum_k C'_kj;  R = softmax_j(col);
//   R' = R / max_j R = exp(col_j - max_j col)   (the softmax denominator cancels);
//   F_sel = lambda * F - (1 - lambda) * R'  over the candidates.
// One workgroup per unit.  The l x l x d contraction runs on the matrix cores for bf16, d = 128;
// a plain vector-ALU kernel covers every other dtype / shape.
#include "gkv_internal.h"
#include <type_traits>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct RedArgs {
  const void* K; const int32_t* d_state; int32_t step; const float* F;
  float lambda, tau, eps; int32_t n_recent; float* R_norm; float* F_sel;
};

// Precision.  A column sum adds up to l cosines and reaches the hundreds, R' = exp(col - max col)
// is compared at 1e-5 relative, and the threshold turns each cosine into a yes/no.  The
// reciprocal norms are formed in fp64.  A column's own norm is a common factor of its whole sum,
// so it is applied once, in fp64, to the finished sum and folded into the threshold (C >= tau
// <=> dot * inv_k >= tau / inv_j); a per-entry fp32 rounding of it would be a systematic error of
// col_j * 1e-7.  What is left per entry in the matrix-core kernel is dot * inv_k in fp32 (dot:
// fp32 accumulation of exact bf16 products; inv_k: the fp64 value rounded once): its error is a
// few 1e-8 of the cosine, random from entry to entry, far inside the 1e-6 band in which a
// threshold decision may legitimately differ from fp64, and it averages out in the sums.  Sums
// run in fp32 over a lane's four entries of a tile pair and in fp64 from there on; exp(col - max)
// is fp64.  The plain kernel does everything in fp64.
__device__ __forceinline__ double block_max_f64(double v, double* red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o));
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmax(fmax(red[0], red[1]), fmax(red[2], red[3]));
}

// Shared tail: R' from the column sums in LDS, then the combination.  cs[j] valid for j < l.
__device__ __forceinline__ void finish_unit(const GkvDims& dm, const RedArgs& a, int unit, int l,
                                            const double* cs, double* red) {
  const int tid = threadIdx.x;
  double mx = -1e300;
  for (int j = tid; j < l; j += 256) mx = fmax(mx, cs[j]);
  mx = block_max_f64(mx, red);
  float* Ru = a.R_norm + (size_t)unit * dm.cap;
  float* Fs = a.F_sel + (size_t)unit * dm.cap;
  const float* Fu = a.F + (size_t)unit * dm.cap;
  const int c = l - dm.w;
  for (int j = tid; j < l; j += 256) {
    const float rn = (float)exp(cs[j] - mx);
    Ru[j] = rn;
    if (j < c) Fs[j] = a.lambda * Fu[j] - (1.f - a.lambda) * rn;
  }
}

// ---- any dtype / shape ------------------------------------------------------------------------
// Dynamic LDS: double cs[cap]; double red[4]; double inv[cap]
template <typename T>
__global__ __launch_bounds__(256) void redundancy_generic_kernel(GkvDims dm, RedArgs a) {
  a.step = resolve_step(dm, a.step);
  extern __shared__ double smem[];
  constexpr int EPC = Elem<T>::EPC;
  const int tid = threadIdx.x, unit = blockIdx.x, lb = unit / dm.Hkv, d = dm.d;
  double* cs = (double*)smem;
  double* red = cs + dm.cap;
  double* inv = red + 4;
  const SeqState st = load_state(a.d_state, lb);
  const int l = compression_length(st, a.step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const T* Kh = (const T*)a.K + (size_t)unit * dm.cap * d;
  for (int n = tid; n < l; n += 256) {
    double ss = 0.0;
    for (int ch = 0; ch < d; ++ch) {
      const double x = (double)Elem<T>::ld(Kh + k_elem_offset<EPC>(n, ch, d, st.n_tiled));
      ss = fma(x, x, ss);
    }
    inv[n] = 1.0 / (sqrt(ss) + (double)a.eps);
  }
  __syncthreads();
  const int first_recent = l - a.n_recent;
  for (int j = tid; j < l; j += 256) {
    double col = 0.0;
    if (j < first_recent) {
      for (int k = 0; k < l; ++k) {
        if (k == j) continue;
        double dot = 0.0;
        for (int ch = 0; ch < d; ++ch)
          dot = fma((double)Elem<T>::ld(Kh + k_elem_offset<EPC>(k, ch, d, st.n_tiled)),
                    (double)Elem<T>::ld(Kh + k_elem_offset<EPC>(j, ch, d, st.n_tiled)), dot);
        const double cv = dot * inv[k] * inv[j];
        if (cv >= (double)a.tau) col += cv;
      }
    }
    cs[j] = col;
  }
  __syncthreads();
  finish_unit(dm, a, unit, l, cs, red);
}

// ---- bf16, d = 128, matrix cores ----------------------------------------------------------------
constexpr int ROW_BYTES = 256;
constexpr int TILE_BYTES = 16 * ROW_BYTES;

__device__ __forceinline__ void load_k_tile(u32x4 (&kA)[4], const char* Kh, int T, int n_tiled,
                                            int lane, int r, int kb) {
  const bool tiled = 16 * T < n_tiled;
  const char* p = Kh + (size_t)T * TILE_BYTES + (tiled ? lane * 16 : r * ROW_BYTES + kb * 16);
  const int step_off = tiled ? 1024 : 64;
#pragma unroll
  for (int c = 0; c < 4; ++c) kA[c] = *(const u32x4*)(p + c * step_off);
}

// A wavefront owns a contiguous quarter of the column tiles and holds NC of them in registers per
// pass; in each pass the workgroup walks all row tiles T together.  The A operand of a tile
// (lane = key + 16*kblock, 8 channels) is also a valid B operand, so C[k, j] = sum_c mfma(A_T[c], A_J[c])
// lands as lane (j = lane%16, blk): rows k = 16T + 4 blk + e.
//
// Row tiles reach the wavefronts through LDS: every wavefront needs every row tile in every pass,
// and if each fetched them itself a unit's keys (l * 256 bytes) would be read 4 * passes times; the
// units resident on one XCD together exceed its L2, so those re-reads would come from memory and
// bound the kernel.  Instead the workgroup moves through the row tiles in groups of four: each
// wavefront fetches one tile of the next group while all four work on the current group, stores it
// into the other half of a two-group ring, and one barrier per group hands the ring over.
//
// Dynamic LDS: double cs[cap]; double red[4]; double inv[cap]; then the ring, 2 groups x 4 tiles x 4 KiB
constexpr int RED_NC = 5;

// Sum over the 16 lanes of a DPP row (lanes 16i .. 16i+15), left in every one of them: lanes ^1
// and ^2 of each quad, then the other quad of each 8 (mirror within 8: all four lanes of a quad
// hold the same value by then), then the other 8 (mirror within 16).  Register-to-register, unlike
// a shuffle through LDS, whose latency four dependent steps per row would pay in full.
__device__ __forceinline__ double row16_sum(double v) {
#define GKV_DPP_STEP(ctrl)                                                                         \
  {                                                                                                \
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), ctrl, 0xF, 0xF, false);       \
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), ctrl, 0xF, 0xF, false);       \
    v += __hiloint2double(hi, lo);                                                                 \
  }
  GKV_DPP_STEP(0xB1)    // quad_perm [1,0,3,2]
  GKV_DPP_STEP(0x4E)    // quad_perm [2,3,0,1]
  GKV_DPP_STEP(0x141)   // row_half_mirror
  GKV_DPP_STEP(0x140)   // row_mirror
#undef GKV_DPP_STEP
  return v;
}
constexpr int RED_RING_BYTES = 2 * 4 * TILE_BYTES;

__global__ __launch_bounds__(256) void redundancy_mfma_kernel(GkvDims dm, RedArgs a) {
  a.step = resolve_step(dm, a.step);
  extern __shared__ double smem[];
  const int tid = threadIdx.x, lane = tid & 63, r = lane & 15, kb = lane >> 4;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int unit = blockIdx.x, lb = unit / dm.Hkv;
  double* cs = (double*)smem;
  double* red = cs + dm.cap;
  double* inv = red + 4;
  char* ring = (char*)(inv + dm.cap);
  const SeqState st = load_state(a.d_state, lb);
  const int l = compression_length(st, a.step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const char* Kh = (const char*)a.K + (size_t)unit * dm.cap * ROW_BYTES;
  const int n_tiles = (l + 15) >> 4;

  constexpr int NC = RED_NC;
  const int per_wave = (n_tiles + 3) >> 2;
  // The column tiles of a pass and this wavefront's tile of the first ring group, requested as
  // early as their registers are free: for pass 0 before the norms (which they do not depend
  // on), for the later passes when the previous pass has used its last row tile.
  u32x4 colA[NC][4], nxt[4];
  auto request_pass = [&](int p) {
    const int J0 = wave * per_wave + p * NC;
#pragma unroll
    for (int cc = 0; cc < NC; ++cc)                         // past the last tile: a clamped duplicate, computed and dropped
      load_k_tile(colA[cc], Kh, min(J0 + cc, n_tiles - 1), st.n_tiled, lane, r, kb);
    load_k_tile(nxt, Kh, min(wave, n_tiles - 1), st.n_tiled, lane, r, kb);
  };
  request_pass(0);

  // Row norms.  Squared norms first, a quarter-wave per row and 16 bytes per lane, eight rows' loads
  // issued together; then one row per thread for the fp64 square root and reciprocal, which cost
  // far more than the sums and would otherwise be repeated by the 16 lanes of every row.
  constexpr int NU = 8;
  for (int n0 = tid >> 4; n0 < n_tiles * 16; n0 += 16 * NU) {
    u32x4 v[NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int n = n0 + 16 * u, ch = tid & 15;
      v[u] = u32x4{0u, 0u, 0u, 0u};
      if (n < l)
        v[u] = *(const u32x4*)((n < st.n_tiled) ? Kh + (size_t)(n >> 4) * TILE_BYTES + ch * 256 + (n & 15) * 16
                                                : Kh + (size_t)n * ROW_BYTES + ch * 16);
    }
#pragma unroll
    for (int u = 0; u < NU; ++u) {
      const int n = n0 + 16 * u;
      double ss = 0.0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const double lo = (double)__uint_as_float(v[u][i] << 16), hi = (double)__uint_as_float(v[u][i] & 0xffff0000u);
        ss = fma(lo, lo, ss);
        ss = fma(hi, hi, ss);
      }
      ss = row16_sum(ss);
      if ((tid & 15) == 0 && n < n_tiles * 16) inv[n] = ss;
    }
  }
  __syncthreads();
  for (int n = tid; n < n_tiles * 16; n += 256) inv[n] = n < l ? 1.0 / (sqrt(inv[n]) + (double)a.eps) : 0.0;
  __syncthreads();

  const int first_recent = l - a.n_recent;
  const double tau = (double)a.tau;
  const int J_end = min(n_tiles, (wave + 1) * per_wave);
  const int n_pass = (per_wave + NC - 1) / NC;          // the same for all wavefronts: they share the barriers below
  const int n_groups = (n_tiles + 3) >> 2;
  // slot of (group parity, tile in group, 16-byte chunk c) for this lane: chunk-major, lane-minor
  auto slot = [&](int par, int u, int c) { return ring + ((par * 4 + u) * 4 + c) * 1024 + lane * 16; };
  auto ring_store = [&](int par, const u32x4 (&t)[4]) {
#pragma unroll
    for (int c = 0; c < 4; ++c) *(u32x4*)slot(par, wave, c) = t[c];
  };
  auto ring_load = [&](u32x4 (&t)[4], int par, int u) {
#pragma unroll
    for (int c = 0; c < 4; ++c) t[c] = *(const u32x4*)slot(par, u, c);
  };

  for (int p = 0; p < n_pass; ++p) {
    const int J0 = wave * per_wave + p * NC;
    double inv_j[NC];
    float thr[NC];
    double col[NC];
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) {
      const int J = min(J0 + cc, n_tiles - 1);
      inv_j[cc] = inv[16 * J + r];
      // C = dot * inv_k * inv_j >= tau  <=>  dot * inv_k >= tau / inv_j: one product per entry, the
      // column's factor applied once to the sum (columns >= l have inv_j = 0 and are dropped below)
      thr[cc] = inv_j[cc] > 0.0 ? (float)(tau / inv_j[cc]) : 3e38f;
      col[cc] = 0.0;
    }
    // One row tile against the NC column tiles.  DIAG: this row tile is one of the column tiles, so
    // the entries with k == j are left out (wavefront-uniform, so the common case carries no test).
    auto row_tile = [&](const u32x4 (&rowA)[4], int T, auto diag) {
      constexpr bool DIAG = decltype(diag)::value;
      const int k0 = 16 * T + 4 * kb;
      float invk[4];                                     // rows >= l have inv = 0: their terms are 0 or fail the test
#pragma unroll
      for (int e = 0; e < 4; ++e) invk[e] = (float)inv[k0 + e];
#pragma unroll
      for (int cc = 0; cc < NC; ++cc) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < 4; ++c)
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, rowA[c]),
                                                        __builtin_bit_cast(bf16x8, colA[cc][c]), acc, 0, 0, 0);
        float part = 0.f;                               // the four entries of this lane, then fp64 across tiles
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float t = acc[e] * invk[e];
          bool pass = t >= thr[cc];
          if (DIAG) pass = pass && !(T == J0 + cc && 4 * kb + e == r);
          part += pass ? t : 0.f;
        }
        col[cc] += (double)part;
      }
    };
    auto row_tile_any = [&](const u32x4 (&rowA)[4], int T) {
      if (T >= J0 && T < J0 + NC) row_tile(rowA, T, std::true_type{});
      else row_tile(rowA, T, std::false_type{});
    };

    ring_store(0, nxt);                                   // group 0 (the previous pass ended with a barrier after its last reads)
    __syncthreads();
    for (int G = 0; G < n_groups; ++G) {
      const int par = G & 1;
      // this wavefront's tile of the next group (clamped past the end: fetched, stored, never used)
      load_k_tile(nxt, Kh, min(4 * (G + 1) + wave, n_tiles - 1), st.n_tiled, lane, r, kb);
      u32x4 row[2][4];
      ring_load(row[0], par, 0);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (u < 3) ring_load(row[(u + 1) & 1], par, u + 1);
        if (4 * G + u < n_tiles) row_tile_any(row[u & 1], 4 * G + u);
      }
      // the other half of the ring was last read in group G - 1, and every wavefront has passed
      // the barrier that ended it
      ring_store(par ^ 1, nxt);
      __syncthreads();
    }
    if (p + 1 < n_pass) request_pass(p + 1);              // travels while the column sums are put together
#pragma unroll
    for (int cc = 0; cc < NC; ++cc) {
      double v = col[cc];
      v += __shfl_xor(v, 16);
      v += __shfl_xor(v, 32);
      const int j = 16 * (J0 + cc) + r;
      if (kb == 0 && J0 + cc < J_end && j < l) cs[j] = j < first_recent ? v * inv_j[cc] : 0.0;
    }
  }
  __syncthreads();
  finish_unit(dm, a, unit, l, cs, red);
}

}  // namespace

hipError_t gkv_launch_redundancy(const GkvLaunch& ln, const GkvDims& dm, int dtype, bool mfma, const void* K,
                                 const int32_t* d_state, int32_t step, const float* F, float lambda, float tau,
                                 float eps, int32_t n_recent, float* R_norm, float* F_sel) {
  RedArgs a{K, d_state, step, F, lambda, tau, eps, n_recent, R_norm, F_sel};
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(double) * (2 * (size_t)dm.cap + 4);
  if (mfma) {
    const size_t with_ring = shmem + RED_RING_BYTES;
    if (with_ring > 64 * 1024) {                         // beyond the default per-workgroup limit: opt in (a CU holds 160 KiB)
      const hipError_t e = hipFuncSetAttribute((const void*)redundancy_mfma_kernel,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)with_ring);
      if (e != hipSuccess) return e;
    }
    return gkv_launch(ln, redundancy_mfma_kernel, dim3(units), dim3(256), with_ring, dm, a);
  }
  if (dtype == GKV_F32)
    return gkv_launch(ln, redundancy_generic_kernel<float>, dim3(units), dim3(256), shmem, dm, a);
  return gkv_launch(ln, redundancy_generic_kernel<uint16_t>, dim3(units), dim3(256), shmem, dm, a);
}

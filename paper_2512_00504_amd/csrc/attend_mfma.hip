// Decode attention on the matrix cores: bf16, head_dim 128, group size g <= 16.
//
// One workgroup of NW wavefronts per (unit, split).  A wavefront owns slices of 16 (or 32) keys
// of the cache (slice it, it + splits*NW, ...) and keeps flash-decoding state (running max,
// running sum, fp32 accumulators) for all g query heads of the KV group, so K and V are read
// from HBM exactly once per KV head.
//
// Per slice and wavefront:
//   K: 16-key tiles.  In the tiled K format each matrix-core A operand (16 keys x 32 channels,
//      lane = key + 16*kblock) is one contiguous 1 KiB load; the few tiles appended since the
//      last compaction are row-major and load as 16 rows x 64 bytes.
//      S^T[key, head] = K[key, :] . Q[head, :]  -> 4 MFMA 16x16x32 per tile.
//      The result lane (head = lane%16, blk = lane/16) holds 4 keys of its head per tile.
//   softmax: running max shared by the 4 lanes of a head (2 cross-lane exchanges), exp2.
//   V: lane (chunk = lane%16, kb = lane/16) loads the 16-byte chunk `chunk` of 4 keys per tile,
//      so a quarter-wave reads one full 256-byte row per load.  An in-register transpose
//      (v_perm_b32) turns that into A operands V^T[channel, key]; with B = P^T[key, head]
//      (the probabilities, already in the right lanes) 8 MFMAs give O^T[channel, head].
// The wavefronts of a workgroup are merged through LDS; splits of one unit are merged by the
// last workgroup to finish (ticket counter), in a fixed order, so results are deterministic.
//
// The newest token's k/v are not read from the cache (another workgroup may be writing that
// row): the lanes that would hold row `len` take them from k_new / v_new instead.
// All stores (output, the appended K/V rows, the window-ring slot) are issued at the end of
// the workgroup and are whole contiguous rows: stores mixed into the read stream, partial-line
// stores and atomics each cost several microseconds per launch on this memory system.
#include "gkv_internal.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int D = 128;
constexpr int ROW_BYTES = D * 2;          // 256
constexpr int TILE_BYTES = 16 * ROW_BYTES;
constexpr int OSTR = D + 4;               // padded LDS row of the per-wave partial outputs
constexpr int PSTR = D + 2;               // split-K partial: o[128], m, l

__device__ __forceinline__ u32x4 ld16(const void* p) { return *(const u32x4*)p; }
// non-temporal load
__device__ __forceinline__ u32x4 ldstream(const void* p) { return __builtin_nontemporal_load((const u32x4*)p); }
__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// One wavefront iteration's loads: KT K tiles (A operands) and 4*KT V rows per lane.
template <int KT>
struct Slice {
  u32x4 kA[KT][4];
  u32x4 vR[4 * KT];
};

// Tiles below n_tiled are in tiled format (lane-contiguous 1 KiB per load); tiles above are
// row-major, where the same operand is 16 rows x 64 bytes per load (only the rows appended since
// the last compaction are in that state).
// K is read with ordinary loads, V with non-temporal loads.  Measured on MI355X with this access
// pattern: both ordinary 67-77% of the HBM peak (worst when K+V exceed the 256 MiB memory-side
// cache), both non-temporal 76%, one stream of each kind 80-85% at every cache size tried (0.3
// to 10 GB), whichever of the two is the non-temporal one.
template <int KT>
__device__ __forceinline__ void issue_slice(Slice<KT>& s, const char* Kh, const char* Vh, int it,
                                            int n_tiled, int lane, int r, int kb) {
  const int key0 = it * 16 * KT;
#pragma unroll
  for (int tt = 0; tt < KT; ++tt) {
    const int row0 = key0 + 16 * tt;
    const char* Kt = Kh + (size_t)(row0 >> 4) * TILE_BYTES;
    const bool tiled = row0 < n_tiled;                     // wave-uniform
    const int lane_off = tiled ? lane * 16 : r * ROW_BYTES + kb * 16;
    const int step_off = tiled ? 1024 : 64;
#pragma unroll
    for (int c = 0; c < 4; ++c) s.kA[tt][c] = ld16(Kt + lane_off + c * step_off);
  }
#pragma unroll
  for (int jj = 0; jj < 4 * KT; ++jj) {
    const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
    s.vR[jj] = ldstream(Vh + (size_t)key * ROW_BYTES + r * 16);
  }
}

// Flash-decoding state of one wavefront: lane (head = lane%16, blk = lane/16) holds the running
// max (in log2 units, shared by the 4 lanes of a head), its partial running sum, and
// O[head][32*blk + 8*e + m] in oacc[m][e].
struct Running {
  float m_run, l_run;
  f32x4 oacc[8];
};

// EDGE = the slice may contain the newest token's row and rows past the end: substitute k/v of
// the newest token from the inputs, mask the rest.  The common path has none of that.
template <int KT, bool EDGE>
__device__ __forceinline__ void process_slice(Slice<KT>& s, Running& st, const bf16x8 (&qB)[4], int it,
                                              float scale_log2, float scale_log2_lo, int r, int kb, bool has_new, int len0,
                                              int n_tot, const char* knew, const char* vnew) {
  // knew / vnew: the newest token's k and v rows, staged in LDS at the start of the workgroup
  constexpr int NS = 4 * KT;
  const int key0 = it * 16 * KT;
  if constexpr (EDGE) {
    if (has_new && key0 <= len0) {
      const int tt_new = (len0 - key0) >> 4, rr = len0 & 15;
#pragma unroll
      for (int tt = 0; tt < KT; ++tt)
        if (tt == tt_new && r == rr) {
#pragma unroll
          for (int c = 0; c < 4; ++c) s.kA[tt][c] = *(const u32x4*)(knew + (4 * c + kb) * 16);
        }
#pragma unroll
      for (int jj = 0; jj < NS; ++jj) {
        const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
        if (key == len0) s.vR[jj] = *(const u32x4*)(vnew + r * 16);
      }
    }
#pragma unroll
    for (int jj = 0; jj < NS; ++jj) {
      const int key = key0 + (jj & 3) + 4 * kb + (jj >> 2) * 16;
      if (key >= n_tot) s.vR[jj] = u32x4{0u, 0u, 0u, 0u};      // stale rows must not reach the MFMA
    }
  }

  // scores: sc[tt][e] = q[head r] . k[key0 + 16 tt + 4 kb + e]
  f32x4 sc[KT];
#pragma unroll
  for (int tt = 0; tt < KT; ++tt) {
    sc[tt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c)
      sc[tt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(s.kA[tt][c]), qB[c], sc[tt], 0, 0, 0);
  }
  float sv[NS];
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    sv[i] = sc[i >> 2][i & 3];
    if constexpr (EDGE) {
      const int key = key0 + (i >> 2) * 16 + 4 * kb + (i & 3);
      if (key >= n_tot) sv[i] = -1e30f;              // finite: -inf times the (signed) low part of the scale would be NaN
    }
  }
  float mx = sv[0];
#pragma unroll
  for (int i = 1; i < NS; ++i) mx = fmaxf(mx, sv[i]);
  mx = fmaxf(mx, __shfl_xor(mx, 16));
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  const float m_new = fmaxf(st.m_run, mx * scale_log2);       // scale > 0: max commutes with it
  if (__any(m_new > st.m_run)) {
    const float corr = __builtin_amdgcn_exp2f(st.m_run - m_new);
    st.l_run *= corr;
#pragma unroll
    for (int m = 0; m < 8; ++m) st.oacc[m] *= corr;
    st.m_run = m_new;
  }
  float pf[NS];
  float psum = 0.f;
#pragma unroll
  for (int i = 0; i < NS; ++i) {
    // exponent of 2 = z * (hi + lo) - m: the window-score kernel forms it identically, so the
    // sums recorded below are the normalisers of its probabilities
    pf[i] = __builtin_amdgcn_exp2f(fmaf(sv[i], scale_log2_lo, fmaf(sv[i], scale_log2, -st.m_run)));
    psum += pf[i];
  }
  st.l_run += psum;

  // O^T[channel 8*(4 blk + e) + m, head] += V^T . P^T; the V^T operands come from an
  // in-register transpose of the lane's [NS keys x 8 channels] block
  if constexpr (KT == 2) {
    f32x8 p8;
#pragma unroll
    for (int i = 0; i < 8; ++i) p8[i] = pf[i];
    const bf16x8 pB = __builtin_convertvector(p8, bf16x8);
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      u32x4 t;
#pragma unroll
      for (int y = 0; y < 4; ++y)
        t[y] = __builtin_amdgcn_perm(s.vR[2 * y + 1][m >> 1], s.vR[2 * y][m >> 1],
                                     (m & 1) ? 0x07060302u : 0x05040100u);
      st.oacc[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(t), pB, st.oacc[m], 0, 0, 0);
    }
  } else {
    f32x4 p4;
#pragma unroll
    for (int i = 0; i < 4; ++i) p4[i] = pf[i];
    const bf16x4 pB4 = __builtin_convertvector(p4, bf16x4);
    const s16x4 pB = __builtin_bit_cast(s16x4, pB4);
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      u32x2 t;
#pragma unroll
      for (int y = 0; y < 2; ++y)
        t[y] = __builtin_amdgcn_perm(s.vR[2 * y + 1][m >> 1], s.vR[2 * y][m >> 1],
                                     (m & 1) ? 0x07060302u : 0x05040100u);
      st.oacc[m] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4, t), pB, st.oacc[m], 0, 0, 0);
    }
  }
}

// KT = 16-key tiles per wavefront iteration (1 or 2)
template <int NW, int KT>
__global__ __launch_bounds__(NW * 64, (KT == 1 && NW <= 8) ? 4 : 2) void attend_mfma_kernel(GkvDims dm, AttendArgs a) {
  a.step = resolve_step(dm, a.step);
  constexpr int KEYS = 16 * KT;             // keys per iteration
  extern __shared__ float smem[];
  __shared__ int s_misc[2];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int r = lane & 15, kb = lane >> 4;
  const int splits = a.splits;
  const int unit = blockIdx.x / splits, sp = blockIdx.x % splits;
  const int j = unit % dm.Hkv, lb = unit / dm.Hkv;
  const int g = dm.g, cap = dm.cap;
  const char* Kh = (const char*)a.K + (size_t)unit * cap * ROW_BYTES;
  const char* Vh = (const char*)a.V + (size_t)unit * cap * ROW_BYTES;
  const int stride = splits * NW;

  // Requests whose addresses do not depend on the state record go out first: the group's
  // queries (B operand of the QK product: lane (head r, kblock kb) holds channels
  // [8*(4c+kb), +8) of q[r]) and the rows stored at the end of the workgroup, one 16-byte piece
  // per thread and round: pieces [0,16) k_new, [16,32) v_new (every workgroup: the wavefront
  // that owns the last slice substitutes them for cache row `len`), [32, 32 + 16 g) the group's
  // q rows for the window ring (split 0 only).
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
  constexpr int AP_ROUNDS = (32 + 16 * 16 + NW * 64 - 1) / (NW * 64);
  u32x4 ap[AP_ROUNDS];
  const bool appender = sp == 0;
  const bool ring_copy = appender && a.copy_q;   // q may already live in its ring slot
  const bool may_grow = a.k_new != nullptr;
  {
    const char* knew_g = (const char*)a.k_new + (size_t)unit * ROW_BYTES;
    const char* vnew_g = (const char*)a.v_new + (size_t)unit * ROW_BYTES;
#pragma unroll
    for (int rd = 0; rd < AP_ROUNDS; ++rd) {
      const int x = tid + rd * NW * 64;
      ap[rd] = u32x4{0u, 0u, 0u, 0u};
      if (x < 16) { if (may_grow) ap[rd] = ld16(knew_g + x * 16); }
      else if (x < 32) { if (may_grow) ap[rd] = ld16(vnew_g + (x - 16) * 16); }
      else if (x < 32 + 16 * g) {
        if (ring_copy) ap[rd] = ld16((const char*)a.q + ((size_t)lb * dm.Hq + j * g) * ROW_BYTES + (x - 32) * 16);
      }
    }
  }

  // The length comes from the state record and the step number; nothing is written back, so
  // the workgroups of a (layer, sequence) need no ordering among themselves.
  const SeqState seq = load_state(a.d_state, lb);
  const int len0 = length_before_step(seq, a.step, cap);
  const bool has_new = may_grow && (len0 < cap);
  const int n_tot = len0 + (has_new ? 1 : 0);
  const float scale_log2 = dm.scale_l2_hi, scale_log2_lo = dm.scale_l2_lo;

  Running st;
  st.m_run = -1e30f;
  st.l_run = 0.f;
#pragma unroll
  for (int m = 0; m < 8; ++m) st.oacc[m] = f32x4{0.f, 0.f, 0.f, 0.f};

  // First slice in flight, then stage k_new / v_new in LDS for whoever owns the last slice.
  const int n_iter = (n_tot + KEYS - 1) / KEYS;
  int it = sp * NW + wave;
  Slice<KT> s;
  if (it < n_iter) issue_slice<KT>(s, Kh, Vh, it, seq.n_tiled, lane, r, kb);
  // stage: 16-byte pieces [0,16) k_new, [16,32) v_new, [32, 32+16g) q rows; kept in LDS, not in
  // registers, until they are stored at the end
  char* stage = (char*)(smem + NW * g * OSTR + NW * 16 + NW * 16);
  const char* knew = stage;
  const char* vnew = stage + ROW_BYTES;
#pragma unroll
  for (int rd = 0; rd < AP_ROUNDS; ++rd) {
    const int x = tid + rd * NW * 64;
    if (x < 32 + 16 * g) *(u32x4*)(stage + x * 16) = ap[rd];
  }
  __syncthreads();
  while (it < n_iter) {
    if ((it + 1) * KEYS > len0) process_slice<KT, true>(s, st, qB, it, scale_log2, scale_log2_lo, r, kb, has_new, len0, n_tot, knew, vnew);
    else process_slice<KT, false>(s, st, qB, it, scale_log2, scale_log2_lo, r, kb, has_new, len0, n_tot, knew, vnew);
    it += stride;
    if (it < n_iter) issue_slice<KT>(s, Kh, Vh, it, seq.n_tiled, lane, r, kb);
  }
  const float m_run = st.m_run, l_run = st.l_run;
  f32x4 (&oacc)[8] = st.oacc;

  // ---- merge the wavefronts of this workgroup -------------------------------------------------
  float* so = smem;                         // [NW][g][OSTR]
  float* sm = so + NW * g * OSTR;           // [NW][16]
  float* sl = sm + NW * 16;                 // [NW][16]
  float l_tot = l_run;                      // the 4 lanes of a head hold partial sums
  l_tot += __shfl_xor(l_tot, 16);
  l_tot += __shfl_xor(l_tot, 32);
  if (r < g) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float* dst = so + (wave * g + r) * OSTR + 32 * kb + 8 * e;
      *(f32x4*)dst = f32x4{oacc[0][e], oacc[1][e], oacc[2][e], oacc[3][e]};
      *(f32x4*)(dst + 4) = f32x4{oacc[4][e], oacc[5][e], oacc[6][e], oacc[7][e]};
    }
    if (kb == 0) { sm[wave * 16 + r] = m_run; sl[wave * 16 + r] = l_tot; }
  }
  __syncthreads();

  // one thread per (head, 4 channels): a single round for g <= 8 with 256 threads
  uint16_t* out = (uint16_t*)a.out + ((size_t)lb * dm.Hq + j * g) * D;
  float* part = a.ws.partials + (size_t)(unit * splits + sp) * g * PSTR;
  for (int x = tid; x < g * 32; x += NW * 64) {
    const int h = x >> 5, c4 = (x & 31) * 4;
    float mw[NW];
    float M = -1e30f;
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) { mw[wv] = sm[wv * 16 + h]; M = fmaxf(M, mw[wv]); }
    float Lsum = 0.f;
    f32x4 o = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int wv = 0; wv < NW; ++wv) {
      const float f = __builtin_amdgcn_exp2f(mw[wv] - M);
      Lsum += sl[wv * 16 + h] * f;
      o += *(const f32x4*)(so + (wv * g + h) * OSTR + c4) * f;
    }
    if (splits == 1) {
      const float inv = Lsum > 0.f ? __builtin_amdgcn_rcpf(Lsum) : 0.f;   // the result is rounded to bf16 anyway
      uint2 packed;
      packed.x = (uint32_t)float_to_bf16_bits(o[0] * inv) | ((uint32_t)float_to_bf16_bits(o[1] * inv) << 16);
      packed.y = (uint32_t)float_to_bf16_bits(o[2] * inv) | ((uint32_t)float_to_bf16_bits(o[3] * inv) << 16);
      *(uint2*)(out + h * D + c4) = packed;
      // softmax statistics of this head's row (running max in log2 units, sum), into the ring slot
      // that also receives q: the window score of the next compression reuses them
      if (c4 == 0 && a.write_stats)
        a.ws.stats[((size_t)(a.step % dm.w) * dm.L * dm.B + lb) * dm.Hq + j * g + h] = make_float2(M, Lsum);
    } else {
      float* ph = part + h * PSTR;
      ph[c4] = o[0]; ph[c4 + 1] = o[1]; ph[c4 + 2] = o[2]; ph[c4 + 3] = o[3];
      if (c4 == 0) { ph[D] = M; ph[D + 1] = Lsum; }
    }
  }

  // ---- append the new row (row-major, one contiguous row each for K and V), push q into the
  //      window ring (contiguous per KV group).  Rows the other workgroups may still be reading
  //      are never the new row's source: they take k_new / v_new from the inputs. ---------------
  if (appender) {
    const int slot = a.step % dm.w;
#pragma unroll
    for (int rd = 0; rd < AP_ROUNDS; ++rd) {
      const int x = tid + rd * NW * 64;
      if (x >= 32 + 16 * g) continue;
      const u32x4 piece = *(const u32x4*)(stage + x * 16);
      if (x < 16) {
        if (has_new) *(u32x4*)((char*)a.K + ((size_t)unit * cap + len0) * ROW_BYTES + x * 16) = piece;
      } else if (x < 32) {
        if (has_new) *(u32x4*)((char*)a.V + ((size_t)unit * cap + len0) * ROW_BYTES + (x - 16) * 16) = piece;
      } else if (ring_copy) {
        *(u32x4*)((char*)a.qwin + ((((size_t)slot * dm.L * dm.B + lb) * dm.Hq + j * g) * ROW_BYTES) + (x - 32) * 16) = piece;
      }
    }
    if (has_new && tid == NW * 64 - 1) a.pos[(size_t)unit * cap + len0] = a.step;
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
}

}  // namespace

template <int NW>
static hipError_t launch_attend(const GkvLaunch& ln, const GkvDims& dm, const AttendArgs& a) {
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(float) * (NW * dm.g * OSTR + NW * 16 + NW * 16) + (32 + 16 * dm.g) * 16;
  if (a.tile_keys == 32 && NW == 4)
    return gkv_launch(ln, attend_mfma_kernel<4, 2>, dim3(units * a.splits), dim3(4 * 64), shmem, dm, a);
  return gkv_launch(ln, attend_mfma_kernel<NW, 1>, dim3(units * a.splits), dim3(NW * 64), shmem, dm, a);
}

hipError_t gkv_launch_attend_mfma(const GkvLaunch& ln, const GkvDims& dm, const AttendArgs& a) {
  if (a.waves == 16) return launch_attend<16>(ln, dm, a);
  if (a.waves == 8) return launch_attend<8>(ln, dm, a);
  return launch_attend<4>(ln, dm, a);
}

// Global-score update, top-(b-w) selection and in-place compaction.  One workgroup of 256
// threads per unit; all score arithmetic in fp32, all index work in integers.
#include "gkv_internal.h"

namespace {

// 16-byte piece as a native vector (arrays of it stay in registers; the runtime's uint4 class does not)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// ---- helpers -------------------------------------------------------------------------------
// Inclusive scan over the 256 threads of a block; `tmp` holds 4 ints of LDS.
__device__ __forceinline__ int block_inclusive_scan(int v, int* tmp) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    int t = __shfl_up(v, o);
    if (lane >= o) v += t;
  }
  __syncthreads();
  if (lane == 63) tmp[wv] = v;
  __syncthreads();
  int add = 0;
  for (int i = 0; i < wv; ++i) add += tmp[i];
  return v + add;
}

// Monotone map float -> uint32 (larger float, larger key); -0 is folded onto +0 first.
__device__ __forceinline__ uint32_t sortable_key(float f) {
  f = f + 0.0f;
  uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// ---- global score (Section 4) --------------------------------------------------------------
__global__ __launch_bounds__(256) void global_update_kernel(GkvDims dm, const float* __restrict__ S,
                                                            const float* __restrict__ F_hist,
                                                            const int32_t* __restrict__ d_state, int step,
                                                            float* __restrict__ F_out) {
  step = resolve_step(dm, step);
  __shared__ float red[8];
  const int unit = blockIdx.x, lb = unit / dm.Hkv, tid = threadIdx.x;
  const SeqState st = load_state(d_state, lb);
  const int l = compression_length(st, step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const int c = l - dm.w;
  int n_hist = st.n_hist;
  n_hist = n_hist < 0 ? 0 : (n_hist > c ? c : n_hist);
  const float* Su = S + (size_t)unit * dm.cap;
  const float* Hu = F_hist + (size_t)unit * dm.cap;
  float* Fu = F_out + (size_t)unit * dm.cap;
  float mx = 0.f;
  for (int n = tid; n < c; n += 256) mx = fmaxf(mx, Su[n]);
  mx = block_max(mx, red);
  for (int n = tid; n < c; n += 256) {
    const float sn = mx > 0.f ? Su[n] / mx : 0.f;
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

// ---- top-(b-w): exact radix select on the float bits, ties to the lower index ---------------
// WITH_UPDATE: F points at the local score S instead, and the kernel first forms the global score
// from it and F_hist exactly as global_update_kernel does (same expressions, same bits), writes
// it to F_out and selects on it: one launch less per compression.
// Dynamic LDS: uint32 keys[cap]
template <bool WITH_UPDATE>
__global__ __launch_bounds__(256) void select_topk_kernel(GkvDims dm, const float* __restrict__ F,
                                                          const float* __restrict__ F_hist,
                                                          const int32_t* __restrict__ d_state, int step,
                                                          float* __restrict__ F_out,
                                                          int32_t* __restrict__ keep_idx) {
  step = resolve_step(dm, step);
  extern __shared__ uint32_t keys[];
  __shared__ int hist[256];
  __shared__ int tmp[4];
  __shared__ int sel[2];
  const int unit = blockIdx.x, lb = unit / dm.Hkv, tid = threadIdx.x;
  const SeqState st = load_state(d_state, lb);
  const int l = compression_length(st, step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const int c = l - dm.w;
  const int k = dm.b - dm.w;                   // c > k because l > b
  const float* Fu = F + (size_t)unit * dm.cap;
  if constexpr (WITH_UPDATE) {
    __shared__ float red[8];
    int n_hist = st.n_hist;
    n_hist = n_hist < 0 ? 0 : (n_hist > c ? c : n_hist);
    const float* Hu = F_hist + (size_t)unit * dm.cap;
    float* Fo = F_out + (size_t)unit * dm.cap;
    float mx = 0.f;
    for (int n = tid; n < c; n += 256) mx = fmaxf(mx, Fu[n]);
    mx = block_max(mx, red);
    for (int n = tid; n < c; n += 256) {
      const float sn = mx > 0.f ? Fu[n] / mx : 0.f;
      float f = sn;
      if (n < n_hist) {
        const float h = dm.alpha * Hu[n];
        f = dm.combine == GKV_COMBINE_MAX ? fmaxf(h, sn)
          : dm.combine == GKV_COMBINE_AVG ? h + (1.f - dm.alpha) * sn
                                          : h + sn;
      }
      Fo[n] = f;
      keys[n] = sortable_key(f);
    }
  } else {
    for (int n = tid; n < c; n += 256) keys[n] = sortable_key(Fu[n]);
  }

  uint32_t prefix = 0, mask = 0;
  int krem = k;
  for (int pass = 3; pass >= 0; --pass) {
    const int shift = 8 * pass;
    hist[tid] = 0;
    __syncthreads();                            // also orders keys[] writes before the first pass
    for (int n = tid; n < c; n += 256) {
      const uint32_t key = keys[n];
      if ((key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    const int v = hist[255 - tid];              // thread t looks at bin 255-t: descending bins
    const int incl = block_inclusive_scan(v, tmp);   // entries in bins >= 255-t
    if (incl >= krem && incl - v < krem) { sel[0] = 255 - tid; sel[1] = krem - (incl - v); }
    __syncthreads();
    prefix |= ((uint32_t)sel[0]) << shift;
    mask |= 255u << shift;
    krem = sel[1];
    __syncthreads();
  }
  // prefix is now the k-th largest key; keep everything above it and the first `krem` equal to it.
  const int per = (c + 255) / 256;
  const int lo = tid * per, hi = min(c, lo + per);
  int n_eq = 0;
  for (int n = lo; n < hi; ++n) n_eq += (keys[n] == prefix);
  int eq_before = block_inclusive_scan(n_eq, tmp) - n_eq;
  int n_keep = 0;
  {
    int eq = eq_before;
    for (int n = lo; n < hi; ++n) {
      const uint32_t key = keys[n];
      if (key > prefix) ++n_keep;
      else if (key == prefix) { n_keep += (eq < krem); ++eq; }
    }
  }
  int out = block_inclusive_scan(n_keep, tmp) - n_keep;
  int32_t* Ku = keep_idx + (size_t)unit * k;
  int eq = eq_before;
  for (int n = lo; n < hi; ++n) {
    const uint32_t key = keys[n];
    bool keep = key > prefix;
    if (key == prefix) { keep = eq < krem; ++eq; }
    if (keep && out < k) Ku[out++] = n;
  }
}

// ---- compaction ----------------------------------------------------------------------------
// grid (units, 2): y = 0 moves K, pos and F_hist; y = 1 moves V (row-major).
// K source rows are in tiled format below the old N_TILED and row-major above; destination rows
// are tiled below nt_new = b rounded down to 16 and row-major above.  Both formats keep a
// 16-row tile inside the same tile-sized block, so the stable-compaction argument still holds
// with chunks that start on tile boundaries: rows are produced in ascending chunks, every
// source piece of a chunk is loaded, then a barrier, then the stores.  Destination index <=
// source index and sources ascend, so a chunk's stores (which stay inside the chunk's tiles)
// never touch a row that a later chunk still has to read.
// State record: every workgroup reads it at its start.  With a ticket array (one counter per
// (layer, sequence), zero between launches) the workgroup that finishes last among the 2 h_kv of
// a (layer, sequence) knows that all of them have read the record, and rewrites it; no data
// depends on that write inside this launch, so the counter needs no fence.  Without a ticket
// array a separate launch rewrites the records.
// Dynamic LDS: int keep_s[b - w]: the kept indices, read from memory once.
template <int PPT>
__global__ __launch_bounds__(256) void compact_kernel(GkvDims dm, int esz, const int32_t* __restrict__ keep_idx,
                                                      const float* __restrict__ F, void* K, void* V,
                                                      float* __restrict__ F_hist, int32_t* pos,
                                                      int32_t* d_state, int step, int32_t* state_ticket) {
  step = resolve_step(dm, step);
  extern __shared__ int keep_s[];
  __shared__ int red_i[4];
  const int unit = blockIdx.x, lb = unit / dm.Hkv, tid = threadIdx.x;
  const bool isK = blockIdx.y == 0;
  const SeqState st = load_state(d_state, lb);
  const int l = compression_length(st, step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const int c = l - dm.w, k = dm.b - dm.w, b = dm.b;
  const int nt_old = st.n_tiled, nt_new = b & ~15;
  const int32_t* Ku = keep_idx + (size_t)unit * k;

  // first destination row whose source differs from it; a K format change rewrites everything
  int first = k;
  for (int n = tid; n < k; n += 256) {
    const int src = Ku[n];
    keep_s[n] = src;
    if (src != n && first == k) first = n;       // ascending per thread: the first hit is its minimum
  }
  for (int o = 32; o > 0; o >>= 1) first = min(first, __shfl_xor(first, o));
  if ((tid & 63) == 0) red_i[tid >> 6] = first;
  __syncthreads();
  first = min(min(red_i[0], red_i[1]), min(red_i[2], red_i[3]));
  if (isK && nt_old != nt_new) first = 0;
  first &= ~15;                                  // chunks start on tile boundaries

  if (isK) {
    float* Hu = F_hist + (size_t)unit * dm.cap;
    const float* Fu = F + (size_t)unit * dm.cap;
    for (int n = tid; n < k; n += 256) {
      int src = keep_s[n];
      src = src < 0 ? 0 : (src >= c ? c - 1 : src);
      Hu[n] = Fu[src];
    }
  }

  const int NP = dm.d * esz / 16;                // 16-byte pieces per row
  int R = (256 * PPT) / NP;                      // rows per chunk: whole tiles, at most one per thread
  R = (R > 256 ? 256 : R) & ~15;
  u32x4* base = (u32x4*)((char*)(isK ? K : V) + (size_t)unit * dm.cap * dm.d * esz);
  int32_t* pu = pos + (size_t)unit * dm.cap;

  // Every load of a round is issued before the first wait: the addresses are computed without
  // branches (pieces beyond the chunk or the budget read row 0, always in bounds, and are not
  // stored), so the PPT 16-byte loads of a thread are in flight together.
  for (int r0 = first; r0 < b; r0 += R) {
    u32x4 buf[PPT];
    int dst[PPT];
#pragma unroll
    for (int i = 0; i < PPT; ++i) {
      const int x = tid + 256 * i;
      const int rr = x / NP, piece = x % NP;
      const int row = r0 + rr;
      const bool valid = rr < R && row < b;
      int src = keep_s[row < k ? row : 0];
      src = row < k ? src : c + (row - k);
      src = src < 0 ? 0 : (src >= l ? l - 1 : src);
      src = valid ? src : 0;
      const int so = (isK && src < nt_old) ? ((src >> 4) * 16 * NP + piece * 16 + (src & 15)) : (src * NP + piece);
      const int d_o = (isK && row < nt_new) ? ((row >> 4) * 16 * NP + piece * 16 + (row & 15)) : (row * NP + piece);
      dst[i] = valid ? d_o : -1;
      buf[i] = base[so];
    }
    const int prow = r0 + tid;
    const bool do_pos = isK && tid < R && prow < b;
    int psrc = keep_s[prow < k ? prow : 0];
    psrc = prow < k ? psrc : c + (prow - k);
    psrc = psrc < 0 ? 0 : (psrc >= l ? l - 1 : psrc);
    const int pos_val = pu[do_pos ? psrc : 0];
    __syncthreads();
#pragma unroll
    for (int i = 0; i < PPT; ++i)
      if (dst[i] >= 0) base[dst[i]] = buf[i];
    if (do_pos) pu[prow] = pos_val;
  }
  // (every wavefront of this workgroup passed the barrier above after reading the record)
  if (state_ticket != nullptr && tid == 0) {
    const int done = atomicAdd(&state_ticket[lb], 1);
    if (done == 2 * dm.Hkv - 1) {
      state_ticket[lb] = 0;
      *(int4*)(d_state + 4 * (size_t)lb) = make_int4(dm.b, step + 1, dm.b - dm.w, dm.b & ~15);
    }
  }
}

// ---- sequence-wise max-pooling of a score over the candidates --------------------------------
// Dynamic LDS: float f[cap]
__global__ __launch_bounds__(256) void pool_scores_kernel(GkvDims dm, const float* __restrict__ F,
                                                          const int32_t* __restrict__ d_state, int step,
                                                          int kernel, float* __restrict__ F_out) {
  step = resolve_step(dm, step);
  extern __shared__ float fbuf[];
  const int unit = blockIdx.x, lb = unit / dm.Hkv, tid = threadIdx.x;
  const int l = compression_length(load_state(d_state, lb), step, dm.b, dm.w, dm.cap);
  if (l == 0) return;
  const int c = l - dm.w, half = kernel / 2;
  const float* Fu = F + (size_t)unit * dm.cap;
  for (int n = tid; n < c; n += 256) fbuf[n] = Fu[n];
  __syncthreads();
  float* Fo = F_out + (size_t)unit * dm.cap;
  for (int n = tid; n < c; n += 256) {
    const int lo = max(0, n - half), hi = min(c - 1, n + half);
    float m = fbuf[lo];
    for (int x = lo + 1; x <= hi; ++x) m = fmaxf(m, fbuf[x]);
    Fo[n] = m;
  }
}

// ---- eviction log: original positions of the candidates that are about to be dropped -------
// A compression from l rows drops l - b of them: s in steady state, up to capacity - b when a
// prompt longer than the budget is compressed, hence capacity - b log entries per unit.
// Dynamic LDS: uint32 kept[cap]
__global__ __launch_bounds__(256) void evicted_positions_kernel(GkvDims dm, const int32_t* __restrict__ keep_idx,
                                                                const int32_t* __restrict__ pos,
                                                                const int32_t* __restrict__ d_state, int step,
                                                                int32_t* __restrict__ evicted) {
  step = resolve_step(dm, step);
  extern __shared__ uint32_t kept[];
  __shared__ int tmp[4];
  const int unit = blockIdx.x, lb = unit / dm.Hkv, tid = threadIdx.x;
  const int n_log = dm.cap - dm.b;
  int32_t* Eu = evicted + (size_t)unit * n_log;
  const int l = compression_length(load_state(d_state, lb), step, dm.b, dm.w, dm.cap);
  if (l == 0) {
    for (int i = tid; i < n_log; i += 256) Eu[i] = -1;
    return;
  }
  const int c = l - dm.w, k = dm.b - dm.w;
  for (int n = tid; n < c; n += 256) kept[n] = 0u;
  __syncthreads();
  const int32_t* Ku = keep_idx + (size_t)unit * k;
  for (int r = tid; r < k; r += 256) {
    const int n = Ku[r];
    if (n >= 0 && n < c) kept[n] = 1u;
  }
  __syncthreads();
  const int per = (c + 255) / 256;
  const int lo = tid * per, hi = min(c, lo + per);
  int n_out = 0;
  for (int n = lo; n < hi; ++n) n_out += (kept[n] == 0u);
  int out = block_inclusive_scan(n_out, tmp) - n_out;
  const int32_t* pu = pos + (size_t)unit * dm.cap;
  for (int n = lo; n < hi; ++n)
    if (kept[n] == 0u && out < n_log) Eu[out++] = pu[n];
  // pad what is left (exactly c - k = l - b rows are dropped when keep_idx holds k distinct candidates)
  const int total = c - k;
  for (int i = total + tid; i < n_log; i += 256) Eu[i] = -1;
}

__global__ void finalize_state_kernel(GkvDims dm, int32_t* d_state, int step) {
  step = resolve_step(dm, step);
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= dm.L * dm.B) return;
  const SeqState st = load_state(d_state, i);
  const int l = compression_length(st, step, dm.b, dm.w, dm.cap);
  if (l > 0) *(int4*)(d_state + 4 * (size_t)i) = make_int4(dm.b, step + 1, dm.b - dm.w, dm.b & ~15);
}

__global__ void add_int_kernel(int32_t* p, int32_t delta) { *p += delta; }

__global__ void fill_zero_kernel(int32_t* p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

}  // namespace

hipError_t gkv_launch_global_update(const GkvLaunch& ln, const GkvDims& dm, const float* S,
                                    const float* F_hist, const int32_t* d_state, int32_t step, float* F_out) {
  const int units = dm.L * dm.B * dm.Hkv;
  return gkv_launch(ln, global_update_kernel, dim3(units), dim3(256), 0, dm, S, F_hist, d_state, (int)step, F_out);
}

hipError_t gkv_launch_select_topk(const GkvLaunch& ln, const GkvDims& dm, const float* F,
                                  const int32_t* d_state, int32_t step, int32_t* keep_idx) {
  const int units = dm.L * dm.B * dm.Hkv;
  return gkv_launch(ln, select_topk_kernel<false>, dim3(units), dim3(256), sizeof(uint32_t) * dm.cap, dm, F,
                    (const float*)nullptr, d_state, (int)step, (float*)nullptr, keep_idx);
}

hipError_t gkv_launch_update_and_select(const GkvLaunch& ln, const GkvDims& dm, const float* S, const float* F_hist,
                                        const int32_t* d_state, int32_t step, float* F_out, int32_t* keep_idx) {
  const int units = dm.L * dm.B * dm.Hkv;
  return gkv_launch(ln, select_topk_kernel<true>, dim3(units), dim3(256), sizeof(uint32_t) * dm.cap, dm, S, F_hist,
                    d_state, (int)step, F_out, keep_idx);
}

hipError_t gkv_launch_compact(const GkvLaunch& ln, const GkvDims& dm, int esz, const int32_t* keep_idx,
                              const float* F, void* K, void* V, float* F_hist, int32_t* pos,
                              int32_t* d_state, int32_t step, int32_t* state_ticket) {
  const int units = dm.L * dm.B * dm.Hkv;
  const size_t shmem = sizeof(int) * (size_t)(dm.b - dm.w);
  const int ppt = ln.ctx ? ln.ctx->compact_ppt : 8;
  auto kern = ppt == 16 ? compact_kernel<16> : ppt == 8 ? compact_kernel<8> : compact_kernel<4>;
  hipError_t e = gkv_launch(ln, kern, dim3(units, 2), dim3(256), shmem, dm, esz, keep_idx, F, K, V,
                            F_hist, pos, d_state, (int)step, state_ticket);
  if (e != hipSuccess || state_ticket != nullptr) return e;
  const int nlb = dm.L * dm.B;
  GkvLaunch plain{ln.ctx, -1, ln.stream};
  return gkv_launch(plain, finalize_state_kernel, dim3((nlb + 255) / 256), dim3(256), 0, dm, d_state, (int)step);
}

hipError_t gkv_launch_pool_scores(const GkvLaunch& ln, const GkvDims& dm, const float* F, const int32_t* d_state,
                                  int32_t step, int32_t kernel, float* F_out) {
  const int units = dm.L * dm.B * dm.Hkv;
  return gkv_launch(ln, pool_scores_kernel, dim3(units), dim3(256), sizeof(float) * dm.cap, dm, F, d_state, (int)step,
                    (int)kernel, F_out);
}

hipError_t gkv_launch_evicted_positions(const GkvLaunch& ln, const GkvDims& dm, const int32_t* keep_idx,
                                        const int32_t* pos, const int32_t* d_state, int32_t step, int32_t* evicted) {
  const int units = dm.L * dm.B * dm.Hkv;
  return gkv_launch(ln, evicted_positions_kernel, dim3(units), dim3(256), sizeof(uint32_t) * dm.cap, dm, keep_idx, pos,
                    d_state, (int)step, evicted);
}

hipError_t gkv_launch_fill_zero(hipStream_t stream, int32_t* p, size_t n) {
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t gkv_launch_add_int(hipStream_t stream, int32_t* p, int32_t delta) {
  hipLaunchKernelGGL(add_int_kernel, dim3(1), dim3(1), 0, stream, p, delta);
  return hipGetLastError();
}

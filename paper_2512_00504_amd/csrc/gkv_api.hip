// C-ABI layer: argument validation, workspace carving, kernel selection, profiling events.
#include <math.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "gkv_internal.h"

// ---- profiling ----------------------------------------------------------------------------------
struct GkvProfile {
  bool on = false;
  struct Rec { hipEvent_t e0, e1; };
  std::vector<Rec> recs[GKV_K_COUNT];
  double done_ms[GKV_K_COUNT] = {};
  int64_t done_n[GKV_K_COUNT] = {};
};

void gkv_profile_events(const GkvLaunch& ln, hipEvent_t* start, hipEvent_t* stop) {
  *start = nullptr; *stop = nullptr;
  GkvProfile* p = ln.ctx ? ln.ctx->prof : nullptr;
  if (!p || !p->on || ln.kernel_id < 0 || ln.kernel_id >= GKV_K_COUNT) return;
  GkvProfile::Rec rec;
  if (hipEventCreate(&rec.e0) != hipSuccess) return;
  if (hipEventCreate(&rec.e1) != hipSuccess) { (void)hipEventDestroy(rec.e0); return; }
  p->recs[ln.kernel_id].push_back(rec);
  *start = rec.e0; *stop = rec.e1;
}

static void profile_drain(GkvProfile* p, int k) {
  for (auto& rec : p->recs[k]) {
    float ms = 0.f;
    if (hipEventSynchronize(rec.e1) == hipSuccess && hipEventElapsedTime(&ms, rec.e0, rec.e1) == hipSuccess) {
      p->done_ms[k] += ms;
      p->done_n[k] += 1;
    }
    (void)hipEventDestroy(rec.e0);
    (void)hipEventDestroy(rec.e1);
  }
  p->recs[k].clear();
}

// ---- context ------------------------------------------------------------------------------------
static gkv_status validate_config(const gkv_config* c) {
  if (!c) return GKV_ERR_INVALID_ARG;
  if (c->dtype != GKV_F32 && c->dtype != GKV_BF16) return GKV_ERR_INVALID_ARG;
  if (c->combine < GKV_COMBINE_MAX || c->combine > GKV_COMBINE_SUM) return GKV_ERR_INVALID_ARG;
  if (c->n_layers < 1 || c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 1)
    return GKV_ERR_INVALID_ARG;
  if (c->n_q_heads % c->n_kv_heads != 0) return GKV_ERR_INVALID_ARG;
  if (c->budget < 2 || c->window < 1 || c->interval < 1) return GKV_ERR_INVALID_ARG;
  if (c->window > c->interval || c->window >= c->budget) return GKV_ERR_INVALID_ARG;
  if (!(c->alpha >= 0.f && c->alpha <= 1.f)) return GKV_ERR_INVALID_ARG;
  if (!(c->softmax_scale >= 0.f) || isinf(c->softmax_scale)) return GKV_ERR_INVALID_ARG;
  const int esz = c->dtype == GKV_F32 ? 4 : 2;
  const int epc = 16 / esz;
  if (c->head_dim % epc != 0 || c->head_dim * esz > 1024) return GKV_ERR_SHAPE;
  if (c->capacity < c->budget + c->interval || c->capacity % 32 != 0 || c->capacity > 4096)
    return GKV_ERR_SHAPE;
  const int64_t units = (int64_t)c->n_layers * c->batch * c->n_kv_heads;
  if (units > (1 << 24)) return GKV_ERR_SHAPE;
  if (gkv_max_lds_bytes(c) > GKV_LDS_LIMIT) return GKV_ERR_SHAPE;
  return GKV_OK;
}

// Largest LDS footprint (dynamic + static, bytes) of any kernel that can be selected for this
// configuration; the plain vector-ALU kernels are included because "force_generic" may select them
// for any shape.  A workgroup gets 64 KiB without opting in to more.
size_t gkv_max_lds_bytes(const gkv_config* c) {
  const size_t cap = (size_t)c->capacity, d = (size_t)c->head_dim;
  const size_t g = (size_t)(c->n_q_heads / c->n_kv_heads);
  size_t need = 16 * (cap + 1 + d);                                 // attend_generic: 4 wavefronts x float[cap + 1 + d]
  auto upd = [&](size_t x) { if (x > need) need = x; };
  upd(4 * (3 * cap + d));                                           // score_generic: at least one wavefront's float[3 cap + d]
  upd(4 * cap + 1024 + 64);                                         // select_topk: keys[cap] + histogram + scan scratch
  upd(16 * cap + 32);                                               // redundancy: double cs[cap], red[4], inv[cap]
  // (the matrix-core redundancy kernel adds a 32 KiB ring of row tiles and asks for the larger
  // per-workgroup allowance itself when that passes 64 KiB: at the largest capacity it needs 96 KiB
  // of the 160 KiB a compute unit holds)
  upd(4 * cap + 64);                                                // pooled score / eviction log
  if (c->dtype == GKV_BF16 && d == 128 && g <= 16)
    upd(4 * (4 * g * 132 + 128) + (32 + 16 * g) * 16 + 16);         // attend_mfma: partial outputs + staged rows
  return need;
}

extern "C" gkv_status gkv_create(const gkv_config* cfg, gkv_ctx** out_ctx) {
  if (!out_ctx) return GKV_ERR_INVALID_ARG;
  *out_ctx = nullptr;
  gkv_status st = validate_config(cfg);
  if (st != GKV_OK) return st;
  gkv_ctx* c = new (std::nothrow) gkv_ctx();
  if (!c) return GKV_ERR_INVALID_ARG;
  c->cfg = *cfg;
  GkvDims& d = c->dims;
  d.L = cfg->n_layers; d.B = cfg->batch; d.Hq = cfg->n_q_heads; d.Hkv = cfg->n_kv_heads;
  d.d = cfg->head_dim; d.g = cfg->n_q_heads / cfg->n_kv_heads;
  d.b = cfg->budget; d.w = cfg->window; d.s = cfg->interval; d.cap = cfg->capacity;
  d.combine = cfg->combine; d.alpha = cfg->alpha;
  d.scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : (float)(1.0 / sqrt((double)cfg->head_dim));
  {
    const double sl2 = (double)d.scale * 1.4426950408889634074;
    d.scale_l2_hi = (float)sl2;
    d.scale_l2_lo = (float)(sl2 - (double)d.scale_l2_hi);
  }
  d.step_base = nullptr;
  c->esz = cfg->dtype == GKV_F32 ? 4 : 2;
  c->attend_splits = 0;
  c->ws_splits = 1;
  c->attend_tile = 16;
  c->force_generic = 0;
  c->reuse_stats = 1;
  c->compact_ppt = 8;
  c->fuse_global = 0;
  c->fuse_select = 1;
  c->attend_waves = 0;
  c->stats_step = new (std::nothrow) int32_t[cfg->window];
  if (!c->stats_step) { delete c; return GKV_ERR_INVALID_ARG; }
  for (int i = 0; i < cfg->window; ++i) c->stats_step[i] = -1;
  c->stats_ws = c->stats_K = c->stats_qwin = nullptr;
  c->mfma_ok = cfg->dtype == GKV_BF16 && d.d == 128 && d.g <= 16;
  c->prof = new (std::nothrow) GkvProfile();
  *out_ctx = c;
  return GKV_OK;
}

extern "C" void gkv_destroy(gkv_ctx* ctx) {
  if (!ctx) return;
  if (ctx->prof) {
    for (int k = 0; k < GKV_K_COUNT; ++k) profile_drain(ctx->prof, k);
    delete ctx->prof;
  }
  delete[] ctx->stats_step;
  delete ctx;
}

extern "C" const char* gkv_status_string(gkv_status st) {
  switch (st) {
    case GKV_OK: return "ok";
    case GKV_ERR_INVALID_ARG: return "invalid argument";
    case GKV_ERR_SHAPE: return "unsupported shape";
    case GKV_ERR_WORKSPACE: return "workspace missing";
    case GKV_ERR_HIP: return "HIP runtime error";
    case GKV_ERR_UNSUPPORTED: return "unsupported";
    case GKV_ERR_OVERFLOW: return "cache capacity exceeded";
    case GKV_ERR_SCRATCH: return "configuration exceeds the static scratch array";
  }
  return "unknown status";
}

static int max_splits(const gkv_ctx* ctx) {
  // a split workgroup of 4 wavefronts covers 128 keys per round
  int m = ctx->dims.cap / 128;
  return m < 1 ? 1 : (m > 64 ? 64 : m);
}

int gkv_effective_splits(const gkv_ctx* ctx) {
  const bool mfma = ctx->mfma_ok && !ctx->force_generic;
  if (!mfma) return 1;
  const int64_t units = (int64_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  int s = ctx->attend_splits;
  (void)units;
  if (s <= 0) s = 1;   // measured: the cross-workgroup merge (device-scope fences over 8 XCDs) costs more than it saves, even at 4 units
  const int m = max_splits(ctx);
  return s > m ? m : s;
}

// Wavefronts per workgroup of the matrix-core attend kernel.  A unit is one workgroup on one CU,
// and a CU pulls only so many bytes per cycle: launches that leave most CUs idle finish sooner
// with 8 wavefronts per unit (measured: 4 to 128 units, 8-16% faster); from a few hundred units
// on 4 and 8 are equal, and 4 keeps the LDS merge small.
static int gkv_attend_waves(const gkv_ctx* ctx) {
  if (ctx->attend_waves > 0) return ctx->attend_waves;
  const int64_t units = (int64_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  const bool fits8 = 8 * ctx->dims.g * 132 * 4 + 8 * 128 + (32 + 16 * ctx->dims.g) * 16 <= 65000;
  return (units <= 256 && fits8 && ctx->attend_tile == 16) ? 8 : 4;
}

static size_t ws_stats_bytes(const gkv_ctx* ctx) {
  return (size_t)ctx->dims.w * ctx->dims.L * ctx->dims.B * ctx->dims.Hq * sizeof(float2);
}

// Split-K partials for `splits` workgroups per unit (none when a unit is not split).
static size_t ws_partials_bytes(const gkv_ctx* ctx, int splits) {
  if (!ctx->mfma_ok || splits <= 1) return 0;
  const size_t units = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  return units * splits * ctx->dims.g * (ctx->dims.d + 2) * sizeof(float);
}

GkvWorkspace gkv_carve_workspace(const gkv_ctx* ctx, void* base) {
  GkvWorkspace w;
  char* p = (char*)base;
  const size_t units = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  w.split_ticket = (int32_t*)p; p += gkv_align256(units * 4);
  w.state_ticket = (int32_t*)p; p += gkv_align256((size_t)ctx->dims.L * ctx->dims.B * 4);
  w.stats = (float2*)p; p += gkv_align256(ws_stats_bytes(ctx));
  w.partials = (float*)p;
  return w;
}

extern "C" gkv_status gkv_workspace_bytes(gkv_ctx* ctx, size_t* out_bytes) {
  if (!ctx || !out_bytes) return GKV_ERR_INVALID_ARG;
  const size_t units = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  // the workspace is sized for the split count in force now; the decode call refuses a larger one
  ctx->ws_splits = gkv_effective_splits(ctx);
  *out_bytes = gkv_align256(units * 4) + gkv_align256((size_t)ctx->dims.L * ctx->dims.B * 4) +
               gkv_align256(ws_stats_bytes(ctx)) +
               gkv_align256(ws_partials_bytes(ctx, ctx->ws_splits)) + 256;
  return GKV_OK;
}

extern "C" gkv_status gkv_workspace_init(gkv_ctx* ctx, void* workspace, void* stream) {
  if (!ctx) return GKV_ERR_INVALID_ARG;
  if (!workspace) return GKV_ERR_WORKSPACE;
  const size_t units = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  const size_t n = (gkv_align256(units * 4) + gkv_align256((size_t)ctx->dims.L * ctx->dims.B * 4)) / 4;   // both ticket arrays
  return gkv_launch_fill_zero((hipStream_t)stream, (int32_t*)workspace, n) == hipSuccess ? GKV_OK : GKV_ERR_HIP;
}

extern "C" gkv_status gkv_cache_bytes(const gkv_config* cfg, int32_t rows, int32_t score_elem_bytes,
                                      size_t* kv_bytes, size_t* score_bytes) {
  if (!cfg || rows < 0 || score_elem_bytes < 1) return GKV_ERR_INVALID_ARG;
  if (cfg->dtype != GKV_F32 && cfg->dtype != GKV_BF16) return GKV_ERR_INVALID_ARG;
  const size_t esz = cfg->dtype == GKV_F32 ? 4 : 2;
  const size_t heads = (size_t)cfg->n_layers * cfg->batch * cfg->n_kv_heads;
  if (kv_bytes) *kv_bytes = heads * (size_t)rows * cfg->head_dim * esz * 2;            // K and V
  if (score_bytes) {
    const int64_t n = (int64_t)cfg->budget - cfg->window;
    *score_bytes = heads * (size_t)(n > 0 ? n : 0) * (size_t)score_elem_bytes;
  }
  return GKV_OK;
}

extern "C" int64_t gkv_k_offset(const gkv_config* cfg, int32_t row, int32_t channel, int32_t n_tiled) {
  if (!cfg || row < 0 || channel < 0 || channel >= cfg->head_dim || n_tiled < 0) return -1;
  const int epc = cfg->dtype == GKV_F32 ? 4 : 8;
  const int64_t d = cfg->head_dim;
  if (row >= (n_tiled & ~15)) return (int64_t)row * d + channel;
  return (int64_t)(row / 16) * 16 * d + (int64_t)(channel / epc) * (16 * epc) + (row % 16) * epc + channel % epc;
}

extern "C" gkv_status gkv_set_param(gkv_ctx* ctx, const char* name, int32_t value) {
  if (!ctx || !name) return GKV_ERR_INVALID_ARG;
  if (!strcmp(name, "attend_splits")) {
    if (value < 0 || value > 64) return GKV_ERR_INVALID_ARG;
    ctx->attend_splits = value;
    return GKV_OK;
  }
  if (!strcmp(name, "attend_tile")) {
    if (value != 16 && value != 32) return GKV_ERR_INVALID_ARG;
    ctx->attend_tile = value;
    return GKV_OK;
  }
  if (!strcmp(name, "force_generic")) { ctx->force_generic = value != 0; return GKV_OK; }
  if (!strcmp(name, "compact_ppt")) {
    if (value != 4 && value != 8 && value != 16) return GKV_ERR_INVALID_ARG;
    ctx->compact_ppt = value;
    return GKV_OK;
  }
  if (!strcmp(name, "attend_waves")) {
    if (value != 0 && value != 4 && value != 8 && value != 16) return GKV_ERR_INVALID_ARG;
    if (value * ctx->dims.g * 132 * 4 + value * 128 + (32 + 16 * ctx->dims.g) * 16 > 65000) return GKV_ERR_SHAPE;
    ctx->attend_waves = value;
    return GKV_OK;
  }
  if (!strcmp(name, "evict_fuse_global")) { ctx->fuse_global = value != 0; return GKV_OK; }
  if (!strcmp(name, "evict_fuse_select")) { ctx->fuse_select = value != 0; return GKV_OK; }
  if (!strcmp(name, "score_reuse_stats")) { ctx->reuse_stats = value != 0; return GKV_OK; }
  return GKV_ERR_INVALID_ARG;
}

// ---- device-side step counter ----------------------------------------------------------------------
extern "C" gkv_status gkv_set_step_base(gkv_ctx* ctx, const int32_t* d_step_base) {
  if (!ctx) return GKV_ERR_INVALID_ARG;
  ctx->dims.step_base = d_step_base;
  for (int i = 0; i < ctx->dims.w; ++i) ctx->stats_step[i] = -1;    // recorded steps were counted from another origin
  return GKV_OK;
}

extern "C" gkv_status gkv_advance_step_base(gkv_ctx* ctx, int32_t delta, void* stream) {
  if (!ctx || !ctx->dims.step_base) return GKV_ERR_INVALID_ARG;
  return gkv_launch_add_int((hipStream_t)stream, const_cast<int32_t*>(ctx->dims.step_base), delta) == hipSuccess
             ? GKV_OK : GKV_ERR_HIP;
}

// ---- the five calls -----------------------------------------------------------------------------
static bool use_mfma_attend(const gkv_ctx* ctx) { return ctx->mfma_ok && !ctx->force_generic; }
static bool use_mfma_score(const gkv_ctx* ctx) {
  return ctx->mfma_ok && !ctx->force_generic && gkv_score_mfma_supported(ctx->dims.g, ctx->dims.w, ctx->dims.cap);
}
static gkv_status check_len(const gkv_ctx* ctx, int32_t len_max_host, bool appending) {
  if (len_max_host < 0) return GKV_ERR_INVALID_ARG;
  if (len_max_host > ctx->dims.cap || (appending && len_max_host >= ctx->dims.cap)) return GKV_ERR_OVERFLOW;
  return GKV_OK;
}
static inline gkv_status hip_status(hipError_t e) { return e == hipSuccess ? GKV_OK : GKV_ERR_HIP; }

// Host bookkeeping of the statistics ring: which decode step each slot's statistics belong to,
// and for which buffers.  Everything is stream-ordered, so "enqueued" is as good as "written".
static void note_stats(gkv_ctx* ctx, int32_t step, bool written, const void* ws, const void* K, const void* qwin) {
  const int w = ctx->dims.w;
  if (ws != ctx->stats_ws || K != ctx->stats_K || qwin != ctx->stats_qwin) {
    for (int i = 0; i < w; ++i) ctx->stats_step[i] = -1;
    ctx->stats_ws = ws; ctx->stats_K = K; ctx->stats_qwin = qwin;
  }
  ctx->stats_step[step % w] = written ? step : -1;
}
static bool stats_cover_window(const gkv_ctx* ctx, int32_t step, const void* ws, const void* K, const void* qwin) {
  const int w = ctx->dims.w;
  if (!ctx->reuse_stats || !ws || ws != ctx->stats_ws || K != ctx->stats_K || qwin != ctx->stats_qwin) return false;
  if (step + 1 < w) return false;
  for (int k = 0; k < w; ++k) {
    const int t = step - w + 1 + k;
    if (ctx->stats_step[t % w] != t) return false;
  }
  return true;
}

extern "C" gkv_status gkv_attend_decode(gkv_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                                        void* K, void* V, int32_t* pos, int32_t step, void* qwin,
                                        const int32_t* d_state, int32_t len_max_host, void* out,
                                        void* workspace, void* stream) {
  if (!ctx || !q || !K || !V || !pos || !qwin || !d_state || !out || step < 0) return GKV_ERR_INVALID_ARG;
  if ((k_new == nullptr) != (v_new == nullptr)) return GKV_ERR_INVALID_ARG;
  if (!workspace) return GKV_ERR_WORKSPACE;
  gkv_status st = check_len(ctx, len_max_host, k_new != nullptr);
  if (st != GKV_OK) return st;
  AttendArgs a{q, k_new, v_new, K, V, pos, step, qwin, d_state, out, gkv_carve_workspace(ctx, workspace), 1,
               ctx->attend_tile, 1, 0, gkv_attend_waves(ctx)};
  {
    const size_t slot_bytes = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hq * ctx->dims.d * ctx->esz;
    a.copy_q = (const char*)q != (const char*)qwin + (size_t)(step % ctx->dims.w) * slot_bytes;
  }
  GkvLaunch ln{ctx, GKV_K_ATTEND, (hipStream_t)stream};
  if (use_mfma_attend(ctx)) {
    a.splits = gkv_effective_splits(ctx);
    if (a.splits > ctx->ws_splits) return GKV_ERR_WORKSPACE;   // partials would not fit the workspace as sized
    // An unsplit appending step leaves (max, sum) of every query head's softmax in the ring slot
    // of this step; the window score can then skip its own pass over the keys for them.
    a.write_stats = a.splits == 1 && k_new != nullptr;
    note_stats(ctx, step, a.write_stats != 0, workspace, K, qwin);
    return hip_status(gkv_launch_attend_mfma(ln, ctx->dims, a));
  }
  note_stats(ctx, step, false, workspace, K, qwin);
  return hip_status(gkv_launch_attend_generic(ln, ctx->dims, ctx->cfg.dtype, a));
}

extern "C" gkv_status gkv_score_window(gkv_ctx* ctx, const void* qwin, const void* K, const int32_t* d_state,
                                       int32_t step, int32_t len_max_host, float* S,
                                       void* workspace, void* stream) {
  if (!ctx || !qwin || !K || !d_state || !S || step < 0) return GKV_ERR_INVALID_ARG;
  gkv_status st = check_len(ctx, len_max_host, false);
  if (st != GKV_OK) return st;
  ScoreArgs a{qwin, K, d_state, step, S, nullptr, nullptr, nullptr};
  GkvLaunch ln{ctx, GKV_K_SCORE, (hipStream_t)stream};
  if (use_mfma_score(ctx)) {
    // Under the causal reading of Eq. 1 a window row's softmax runs over exactly the keys its
    // query attended to when it was decoded: if the last w decode calls on these buffers were the
    // window's steps, their recorded (max, sum) are the row statistics and one pass suffices.
    if (stats_cover_window(ctx, step, workspace, K, qwin)) a.stats = gkv_carve_workspace(ctx, workspace).stats;
    return hip_status(gkv_launch_score_mfma(ln, ctx->dims, a));
  }
  return hip_status(gkv_launch_score_generic(ln, ctx->dims, ctx->cfg.dtype, a));
}

extern "C" gkv_status gkv_global_update(gkv_ctx* ctx, const float* S, const float* F_hist,
                                        const int32_t* d_state, int32_t step, int32_t len_max_host,
                                        float* F_out, void* stream) {
  if (!ctx || !S || !F_hist || !d_state || !F_out || step < 0) return GKV_ERR_INVALID_ARG;
  gkv_status st = check_len(ctx, len_max_host, false);
  if (st != GKV_OK) return st;
  GkvLaunch ln{ctx, GKV_K_GLOBAL, (hipStream_t)stream};
  return hip_status(gkv_launch_global_update(ln, ctx->dims, S, F_hist, d_state, step, F_out));
}

extern "C" gkv_status gkv_select_topk(gkv_ctx* ctx, const float* F, const int32_t* d_state, int32_t step,
                                      int32_t len_max_host, int32_t* keep_idx, void* workspace, void* stream) {
  (void)workspace;
  if (!ctx || !F || !d_state || !keep_idx || step < 0) return GKV_ERR_INVALID_ARG;
  gkv_status st = check_len(ctx, len_max_host, false);
  if (st != GKV_OK) return st;
  GkvLaunch ln{ctx, GKV_K_TOPK, (hipStream_t)stream};
  return hip_status(gkv_launch_select_topk(ln, ctx->dims, F, d_state, step, keep_idx));
}

extern "C" gkv_status gkv_compact(gkv_ctx* ctx, const int32_t* keep_idx, const float* F, void* K, void* V,
                                  float* F_hist, int32_t* pos, int32_t* d_state, int32_t step,
                                  void* workspace, void* stream) {
  if (!ctx || !keep_idx || !F || !K || !V || !F_hist || !pos || !d_state || step < 0) return GKV_ERR_INVALID_ARG;
  if (F == F_hist) return GKV_ERR_INVALID_ARG;
  GkvLaunch ln{ctx, GKV_K_COMPACT, (hipStream_t)stream};
  // with a workspace the last compaction workgroup of a (layer, sequence) rewrites its state
  // record; without one a second small launch does
  int32_t* ticket = workspace ? gkv_carve_workspace(ctx, workspace).state_ticket : nullptr;
  return hip_status(gkv_launch_compact(ln, ctx->dims, ctx->esz, keep_idx, F, K, V, F_hist, pos, d_state, step, ticket));
}

extern "C" gkv_status gkv_evict(gkv_ctx* ctx, const void* qwin, void* K, void* V, float* F_hist, int32_t* pos,
                                int32_t* d_state, int32_t step, int32_t len_max_host,
                                float* S, float* F, int32_t* keep_idx, void* workspace, void* stream) {
  if (!ctx || !qwin || !K || !V || !F_hist || !pos || !d_state || !S || !F || !keep_idx || step < 0)
    return GKV_ERR_INVALID_ARG;
  if (F == F_hist) return GKV_ERR_INVALID_ARG;
  gkv_status st = check_len(ctx, len_max_host, false);
  if (st != GKV_OK) return st;
  if (ctx->fuse_global && use_mfma_score(ctx)) {
    // local and global score in one launch: the score kernel keeps S in LDS and finishes with the update
    ScoreArgs a{qwin, K, d_state, step, S, nullptr, F_hist, F};
    if (stats_cover_window(ctx, step, workspace, K, qwin)) a.stats = gkv_carve_workspace(ctx, workspace).stats;
    GkvLaunch ln{ctx, GKV_K_SCORE, (hipStream_t)stream};
    st = hip_status(gkv_launch_score_mfma(ln, ctx->dims, a));
    if (st != GKV_OK) return st;
  } else {
    st = gkv_score_window(ctx, qwin, K, d_state, step, len_max_host, S, workspace, stream);
    if (st != GKV_OK) return st;
    if (ctx->fuse_select) {
      // the global score is formed at the head of the selection kernel (same arithmetic as
      // gkv_global_update, F written as well): one launch less per compression
      GkvLaunch ln{ctx, GKV_K_TOPK, (hipStream_t)stream};
      st = hip_status(gkv_launch_update_and_select(ln, ctx->dims, S, F_hist, d_state, step, F, keep_idx));
      if (st != GKV_OK) return st;
      return gkv_compact(ctx, keep_idx, F, K, V, F_hist, pos, d_state, step, workspace, stream);
    }
    st = gkv_global_update(ctx, S, F_hist, d_state, step, len_max_host, F, stream);
    if (st != GKV_OK) return st;
  }
  st = gkv_select_topk(ctx, F, d_state, step, len_max_host, keep_idx, workspace, stream);
  if (st != GKV_OK) return st;
  return gkv_compact(ctx, keep_idx, F, K, V, F_hist, pos, d_state, step, workspace, stream);
}

// ---- compression for callers that cannot allocate ---------------------------------------------
// The intermediates of one compression (S, F, keep_idx) live in a fixed array in device memory
// that every GPU the library runs on holds until the process ends.  In host code the array's
// name is only a handle for hipGetSymbolAddress; the address that kernels and copies use is the
// one that call returns, looked up once per device.
static __device__ __align__(256) unsigned char scratch[GKV_STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {};

static gkv_status static_scratch_of_current_device(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return GKV_ERR_HIP;
  if (dev < 0 || dev >= 64) return GKV_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GKV_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = (char*)g_scratch_ptr[dev];
  return GKV_OK;
}

extern "C" gkv_status gkv_evict_static(gkv_ctx* ctx, const void* qwin, void* K, void* V, float* F_hist,
                                       int32_t* pos, int32_t* d_state, int32_t step, int32_t len_max_host,
                                       void* workspace, void* stream) {
  if (!ctx || !qwin || !K || !V || !F_hist || !pos || !d_state || step < 0) return GKV_ERR_INVALID_ARG;
  const size_t units = (size_t)ctx->dims.L * ctx->dims.B * ctx->dims.Hkv;
  const size_t score_bytes = gkv_align256(units * ctx->dims.cap * sizeof(float));
  const size_t keep_bytes = gkv_align256(units * (size_t)(ctx->dims.b - ctx->dims.w) * sizeof(int32_t));
  if (2 * score_bytes + keep_bytes > (size_t)GKV_STATIC_SCRATCH_BYTES) return GKV_ERR_SCRATCH;
  char* base = nullptr;
  gkv_status st = static_scratch_of_current_device(&base);
  if (st != GKV_OK) return st;
  float* S = (float*)base;
  float* F = (float*)(base + score_bytes);
  int32_t* keep_idx = (int32_t*)(base + 2 * score_bytes);
  return gkv_evict(ctx, qwin, K, V, F_hist, pos, d_state, step, len_max_host, S, F, keep_idx, workspace, stream);
}

extern "C" gkv_status gkv_redundancy_combine(gkv_ctx* ctx, const void* K, const int32_t* d_state, int32_t step,
                                             int32_t len_max_host, const float* F, float lambda, float tau,
                                             float eps, int32_t n_recent, float* R_norm, float* F_sel,
                                             void* workspace, void* stream) {
  (void)workspace;
  if (!ctx || !K || !d_state || !F || !R_norm || !F_sel || step < 0) return GKV_ERR_INVALID_ARG;
  if (!(lambda >= 0.f && lambda <= 1.f) || !(tau > -1.5f && tau < 1.5f) || !(eps >= 0.f) || n_recent < 0)
    return GKV_ERR_INVALID_ARG;
  if (F == F_sel) return GKV_ERR_INVALID_ARG;
  gkv_status st = check_len(ctx, len_max_host, false);
  if (st != GKV_OK) return st;
  GkvLaunch ln{ctx, GKV_K_REDUNDANCY, (hipStream_t)stream};
  return hip_status(gkv_launch_redundancy(ln, ctx->dims, ctx->cfg.dtype, use_mfma_attend(ctx), K, d_state, step, F,
                                          lambda, tau, eps, n_recent, R_norm, F_sel));
}

extern "C" gkv_status gkv_pool_scores(gkv_ctx* ctx, const float* F, const int32_t* d_state, int32_t step,
                                      int32_t kernel, float* F_out, void* stream) {
  if (!ctx || !F || !d_state || !F_out || step < 0 || kernel < 1 || F == F_out) return GKV_ERR_INVALID_ARG;
  GkvLaunch ln{ctx, -1, (hipStream_t)stream};
  return hip_status(gkv_launch_pool_scores(ln, ctx->dims, F, d_state, step, kernel, F_out));
}

extern "C" gkv_status gkv_evicted_positions(gkv_ctx* ctx, const int32_t* keep_idx, const int32_t* pos,
                                            const int32_t* d_state, int32_t step, int32_t* evicted, void* stream) {
  if (!ctx || !keep_idx || !pos || !d_state || !evicted || step < 0) return GKV_ERR_INVALID_ARG;
  GkvLaunch ln{ctx, -1, (hipStream_t)stream};
  return hip_status(gkv_launch_evicted_positions(ln, ctx->dims, keep_idx, pos, d_state, step, evicted));
}

// ---- profiling API ------------------------------------------------------------------------------
extern "C" gkv_status gkv_profile_enable(gkv_ctx* ctx, int32_t on) {
  if (!ctx || !ctx->prof) return GKV_ERR_INVALID_ARG;
  ctx->prof->on = on != 0;
  return GKV_OK;
}
extern "C" gkv_status gkv_profile_read(gkv_ctx* ctx, int32_t kernel_id, double* total_ms, int64_t* launches) {
  if (!ctx || !ctx->prof || kernel_id < 0 || kernel_id >= GKV_K_COUNT) return GKV_ERR_INVALID_ARG;
  profile_drain(ctx->prof, kernel_id);
  if (total_ms) *total_ms = ctx->prof->done_ms[kernel_id];
  if (launches) *launches = ctx->prof->done_n[kernel_id];
  return GKV_OK;
}
extern "C" gkv_status gkv_profile_reset(gkv_ctx* ctx) {
  if (!ctx || !ctx->prof) return GKV_ERR_INVALID_ARG;
  for (int k = 0; k < GKV_K_COUNT; ++k) {
    profile_drain(ctx->prof, k);
    ctx->prof->done_ms[k] = 0;
    ctx->prof->done_n[k] = 0;
  }
  return GKV_OK;
}

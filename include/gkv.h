/*
 * gkv.h - C ABI of the G-KV decode/evict hot path for AMD MI355X (gfx950).
 *
 * Per layer and decode step the path is: attention of the newest query over a
 * budget-capped KV cache; every s steps, the local score of each cached token
 * from the observation window (paper: Preliminary, Eq. 1 and Eq. 2), the
 * global score that merges it with the token's decayed history (paper:
 * Section 4, the max / average / summation forms), top-(b-w) selection per
 * KV head and compaction of K, V and the recorded scores.
 *
 * Notation (paper, Preliminary): h_q query heads, h_kv KV heads, g = h_q/h_kv,
 * d head dim, l cache length, b budget, w observation window, s compression
 * interval, alpha memory-decay rate.  Query head i reads KV head i / g.
 * A "unit" is one (layer, sequence, KV head).  L = n_layers, B = batch.
 *
 * Conventions for every call
 *   - All data pointers are DEVICE pointers owned by the caller; the library
 *     never allocates or frees device memory.  `workspace` is device memory of
 *     at least gkv_workspace_bytes() bytes, zeroed once with
 *     gkv_workspace_init() and then left to the library.
 *   - `stream` is a hipStream_t passed as void*; calls only enqueue work on it
 *     and return.  No host synchronisation, no device-to-host copies.  Lengths
 *     live on the device (d_state); `len_max_host` is only an upper bound the
 *     host knows, used to size launches and to reject overflow.
 *   - d_state is int32 [L,B,4], one record per (layer, sequence):
 *       [GKV_ST_LEN]      cache length before decode step [GKV_ST_LEN_STEP];
 *       [GKV_ST_LEN_STEP] the step that length refers to.  Every decode step
 *                         appends one row, so before step t >= LEN_STEP the length
 *                         is LEN + (t - LEN_STEP).  The decode kernel therefore never
 *                         writes a length: no atomics, no ordering between its
 *                         workgroups.  Compaction rewrites the pair.
 *       [GKV_ST_N_HIST]   leading rows that carry a recorded global score.
 *       [GKV_ST_N_TILED]  leading rows of K stored in tiled format (multiple of 16).
 *     A fresh sequence is {prompt_len, first_step, 0, 0}.
 *   - Arrays are row-major with the last index contiguous, base pointers 16-byte
 *     aligned.  Element type of q, k_new, v_new, K, V, qwin, out is
 *     config.dtype; scores are float; lengths, positions, indices are int32.
 *   - K cache layout: each KV head's [capacity, d] block is a sequence of 16-row
 *     tiles of 16*d elements.  Rows at or above N_TILED are plain row-major
 *     (element (n, c) at n*d + c): that is how appended rows are written, one
 *     contiguous row per step.  Rows below N_TILED are in tiled format: inside
 *     their tile the 16-byte chunks are chunk-major, element (n, c) at
 *         (n/16)*16*d + (c/E)*16*E + (n%16)*E + c%E,   E = 16/sizeof(element),
 *     which makes a wavefront's matrix-core operand load of a 16-key tile one
 *     contiguous 1 KiB read.  Compaction writes the kept rows in tiled format
 *     (N_TILED = budget rounded down to 16).  A row-major K cache with
 *     N_TILED = 0 is a valid state.  gkv_k_offset() returns the offset.
 *     V is plain row-major [capacity, d].
 *   - A context keeps host-side bookkeeping (tuning knobs, which ring slots hold recorded
 *     softmax statistics): use it from one thread at a time, one context per set of buffers.
 *   - Return value: GKV_OK or an error code; arguments are validated on the
 *     host before anything is enqueued, a failed call enqueues nothing.
 *     Results are deterministic: same inputs, same bits.
 *   - A compression call is a no-op for every (layer, sequence) whose length is
 *     not above the budget, so ragged batches are legal.  It is also a no-op while
 *     fewer than w steps have been decoded since LEN_STEP (the observation window
 *     consists of generated tokens: a prompt loaded as {prompt_len, first_step, 0, 0}
 *     brings keys and values but no window queries, so the ring slots are not yet
 *     all written).  In a batch every sequence shares the step counter; a sequence
 *     with a shorter prompt simply starts with a shorter cache.
 */
#ifndef GKV_H
#define GKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GKV_OK = 0,
  GKV_ERR_INVALID_ARG = 1,   /* null pointer, bad enum, alpha outside [0,1], w > s, w >= b ... */
  GKV_ERR_SHAPE = 2,         /* shape the kernels do not support (see gkv_create) */
  GKV_ERR_WORKSPACE = 3,     /* workspace pointer missing, or sized for fewer attend_splits */
  GKV_ERR_HIP = 4,           /* a HIP runtime call failed */
  GKV_ERR_UNSUPPORTED = 5,
  GKV_ERR_OVERFLOW = 6,      /* len_max_host would exceed the capacity */
  GKV_ERR_SCRATCH = 7        /* configuration too large for the fixed scratch array of gkv_evict_static */
} gkv_status;

typedef enum { GKV_F32 = 0, GKV_BF16 = 1 } gkv_dtype;

/* Section 4: the three forms of the global score. */
typedef enum { GKV_COMBINE_MAX = 0, GKV_COMBINE_AVG = 1, GKV_COMBINE_SUM = 2 } gkv_combine;

typedef struct gkv_config {
  int32_t n_layers, batch;          /* L, B */
  int32_t n_q_heads, n_kv_heads;    /* h_q, h_kv; h_q % h_kv == 0 */
  int32_t head_dim;                 /* d; multiple of 16/sizeof(element), at most 1024 bytes per row */
  int32_t budget, window, interval; /* b, w, s;  w <= s, w < b */
  int32_t capacity;                 /* rows per KV head; >= b + s, multiple of 32, at most 4096 and small
                                       enough for every kernel's 64 KiB of LDS: 16*(capacity+1+d) bytes
                                       (plain attend kernel) and 16*capacity+32 (redundancy score) */
  int32_t dtype;                    /* gkv_dtype */
  int32_t combine;                  /* gkv_combine */
  float alpha;                      /* memory-decay rate in [0,1]; 0 = local score only */
  float softmax_scale;              /* 0 means 1/sqrt(d) as in Eq. 1 */
} gkv_config;

enum { GKV_ST_LEN = 0, GKV_ST_LEN_STEP = 1, GKV_ST_N_HIST = 2, GKV_ST_N_TILED = 3, GKV_ST_FIELDS = 4 };

typedef struct gkv_ctx gkv_ctx;     /* opaque, host memory only */

/* Validates the configuration and builds a host-side context.  Touches no GPU. */
gkv_status gkv_create(const gkv_config* cfg, gkv_ctx** out_ctx);
void gkv_destroy(gkv_ctx* ctx);
const char* gkv_status_string(gkv_status st);

/* Bytes of device workspace the calls below need for this context with the tuning knobs as they
 * are now; the context remembers the "attend_splits" value the size covers, and
 * gkv_attend_decode returns GKV_ERR_WORKSPACE if the knob was raised afterwards. */
gkv_status gkv_workspace_bytes(gkv_ctx* ctx, size_t* out_bytes);
/* Enqueues a fill kernel that zeroes the workspace's counters (one per unit, used when a
 * unit's attention is split over several workgroups; one per (layer, sequence), used by the
 * compaction to find the workgroup that finishes last).  The kernels leave them at zero.
 * Call once, before the first call that takes the workspace. */
gkv_status gkv_workspace_init(gkv_ctx* ctx, void* workspace, void* stream);

/* Host-only helpers.
 * gkv_cache_bytes: bytes of K+V cache and of the score cache F for the whole
 * configuration at `rows` rows per KV head (paper, appendix "Memory Analysis":
 * rows = b + s for the KV cache between compressions, b - w scores per head).
 * gkv_k_offset: element offset of (row, channel) inside one KV head's K block when
 * the first n_tiled rows are in tiled format. */
gkv_status gkv_cache_bytes(const gkv_config* cfg, int32_t rows, int32_t score_elem_bytes,
                           size_t* kv_bytes, size_t* score_bytes);
int64_t gkv_k_offset(const gkv_config* cfg, int32_t row, int32_t channel, int32_t n_tiled);

/* Tuning knobs (host only): "attend_splits" (workgroups per unit in the matrix-core
 * attend kernel; 0 = default = 1; set it before gkv_workspace_bytes), "attend_tile" (16 or 32 keys per wavefront iteration of
 * the matrix-core attend kernel), "attend_waves" (4, 8 or 16 wavefronts per workgroup of that
 * kernel; 0 = default: 8 for launches of at most 256 units, else 4), "force_generic" (1 = use the plain vector-ALU
 * kernels even where matrix-core kernels exist), "compact_ppt" (4, 8 or 16: 16-byte pieces
 * a thread of the compaction kernel keeps in flight per round), "score_reuse_stats" (0 = the
 * window score always computes its rows' softmax statistics itself instead of reusing the
 * ones the matrix-core decode kernel recorded during the window's decode steps; see
 * gkv_score_window), "evict_fuse_global" (1 = gkv_evict computes the global score in the tail
 * of the matrix-core window-score kernel, S still in LDS, instead of a launch of its own;
 * same results, measured neither faster nor slower), "evict_fuse_select" (default 1: gkv_evict
 * forms the global score at the head of the selection kernel, one launch less per compression;
 * 0 = a launch of its own as in gkv_global_update; same bits either way). */
gkv_status gkv_set_param(gkv_ctx* ctx, const char* name, int32_t value);

/*
 * Device-side step counter, for callers that record the calls once and replay them (HIP
 * graphs): the host arguments of a recorded launch are frozen, so the step number must come
 * from device memory.  With a step base set, the `step` argument of every call below is
 * relative and the kernels use *d_step_base + step.  d_step_base is one int32 of device memory,
 * the caller's; NULL switches back to absolute steps.  gkv_advance_step_base enqueues
 * *d_step_base += delta (a one-thread kernel, recordable).  Whenever a call is enqueued or
 * replayed the base must be a multiple of both w and s (so that ring slots and triggers computed
 * from the relative step on the host match the device's); advance it by whole compression cycles.
 * len_max_host stays a host bound: in a recorded steady-state cycle it is b + i for the i-th step.
 * Every call only launches kernels, so all of them can be recorded; gkv_workspace_init and the
 * first gkv_evict_static on a device should run before recording starts.
 */
gkv_status gkv_set_step_base(gkv_ctx* ctx, const int32_t* d_step_base);
gkv_status gkv_advance_step_base(gkv_ctx* ctx, int32_t delta, void* stream);

/*
 * Every decode step (paper, Preliminary: the cache the newest token attends to;
 * evicted entries are invisible to later tokens).  For every (layer, sequence),
 * with len = LEN + (step - LEN_STEP) from d_state:
 *   attends q over rows [0, len) plus the new row (k_new, v_new):
 *   out[i] = softmax(q[i] . K[i/g]^T * scale) V[i/g]; writes k_new, v_new as row
 *   len of K (row-major) and V, pos[len] = step, and q into slot step % w of the
 *   window ring qwin.  With k_new == v_new == NULL nothing is appended and the
 *   attention covers rows [0, len) only.  d_state is not written.
 * q, out [L,B,h_q,d]; k_new, v_new [L,B,h_kv,d]; K, V [L,B,h_kv,capacity,d];
 * pos [L,B,h_kv,capacity]; qwin [w,L,B,h_q,d]: slot step % w is one whole q tensor.
 * If q already IS that slot (q == qwin + (step % w) * L*B*h_q*d elements: the
 * producer of q wrote it into the ring), nothing is copied.  len_max_host: host
 * bound with every len <= len_max_host < capacity.
 */
gkv_status gkv_attend_decode(gkv_ctx* ctx, const void* q, const void* k_new, const void* v_new,
                             void* K, void* V, int32_t* pos, int32_t step, void* qwin,
                             const int32_t* d_state, int32_t len_max_host, void* out,
                             void* workspace, void* stream);

/*
 * The four compression calls take `step`, the index of the latest decode step;
 * the length they see is l = LEN + (step + 1 - LEN_STEP).
 *
 * Local score (paper, Preliminary, Eq. 1 then group max-reduce then Eq. 2).
 * With c = l - w: window row k is the query decoded at step step - w + 1 + k
 * (its ring slot), normalised over rows [0, c + k] (the keys it saw when decoded);
 * S[n] = (1/w) sum_k max_{heads of the group} A[head, k, n] for the candidates
 * n < c.  Entries n >= c are not written.  S [L,B,h_kv,capacity].
 * Under this reading a window row's softmax runs over exactly the keys its query attended to
 * when it was decoded.  The matrix-core decode kernel therefore records every query head's
 * (max, sum) in the workspace, and when the last w gkv_attend_decode calls on this context
 * with these same K, qwin and workspace pointers were the steps step-w+1 .. step (each
 * appending a row), this call takes the rows' statistics from there and reads K once instead
 * of twice.  Otherwise it computes them itself.  The caller must not change K rows or ring
 * slots between those decode calls and this one (or sets "score_reuse_stats" to 0).
 */
gkv_status gkv_score_window(gkv_ctx* ctx, const void* qwin, const void* K, const int32_t* d_state,
                            int32_t step, int32_t len_max_host, float* S,
                            void* workspace, void* stream);

/*
 * Global score (paper, Section 4).  Sn = S / max_{n<c} S per KV head;
 * F_out[n] = combine(alpha * F_hist[n], Sn[n]) for n < N_HIST, else Sn[n].
 * combine is max, alpha*F + (1-alpha)*Sn, or alpha*F + Sn.  A zero maximum
 * gives Sn = 0.  S, F_hist, F_out [L,B,h_kv,capacity].
 */
gkv_status gkv_global_update(gkv_ctx* ctx, const float* S, const float* F_hist,
                             const int32_t* d_state, int32_t step, int32_t len_max_host,
                             float* F_out, void* stream);

/*
 * Top-(b-w) selection per unit (paper, Preliminary and Section 4): ascending
 * indices of the b-w largest F among candidates [0, l-w); equal scores: lower
 * index first.  keep_idx [L,B,h_kv,b-w].  Always writes valid in-range indices,
 * whatever the score bits.
 */
gkv_status gkv_select_topk(gkv_ctx* ctx, const float* F, const int32_t* d_state, int32_t step,
                           int32_t len_max_host, int32_t* keep_idx, void* workspace, void* stream);

/*
 * Compaction (paper, Section 4: the kept entries' scores are recorded for the
 * next compression; appendix "Memory Analysis": cache of b rows, b-w scores).
 * In place and stable: row keep_idx[r] moves to r for r < b-w (K, V, pos),
 * F_hist[r] = F[keep_idx[r]], the w window rows [l-w, l) move to [b-w, b).  K rows
 * below b rounded down to 16 are written in tiled format.  Then d_state becomes
 * {b, step + 1, b - w, b rounded down to 16}.  F must not alias F_hist.
 * workspace may be NULL: the state records are then rewritten by a second small launch
 * instead of by the last workgroup of each (layer, sequence).
 */
gkv_status gkv_compact(gkv_ctx* ctx, const int32_t* keep_idx, const float* F, void* K, void* V,
                       float* F_hist, int32_t* pos, int32_t* d_state, int32_t step,
                       void* workspace, void* stream);

/*
 * Redundancy score and its combination with the global score (paper, appendix
 * "Integrating the Global Score with Other Methods"; the paper's "G-KV" is the
 * max-form global score with this term).  Per KV head, over the l cached keys:
 * Kn = K/(||K||_2 + eps), C = Kn Kn^T, entries below tau are zeroed, and so are
 * the diagonal and the columns of the n_recent newest rows (the paper gives no
 * values for these: caller's parameters); col_j = sum_k C'_kj; R = softmax_j col;
 * R_norm = R / max_j R; F_sel[n] = lambda*F[n] - (1-lambda)*R_norm[n] for the
 * candidates n < l-w.  Call it between gkv_global_update and gkv_select_topk,
 * select on F_sel, and pass F (not F_sel) to gkv_compact: the recorded history
 * stays the global score.  R_norm, F_sel [L,B,h_kv,capacity]; F_sel must not alias F.
 */
gkv_status gkv_redundancy_combine(gkv_ctx* ctx, const void* K, const int32_t* d_state, int32_t step,
                                  int32_t len_max_host, const float* F, float lambda, float tau,
                                  float eps, int32_t n_recent, float* R_norm, float* F_sel,
                                  void* workspace, void* stream);

/*
 * SnapKV-style plug-in (paper, same appendix): sequence-wise max-pooling of a score over
 * the candidates, F_out[n] = max F[m] for |m - n| <= kernel/2, clipped at the ends.  The
 * paper gives no kernel size (caller's parameter).  Select on F_out, record F.
 * F_out must not alias F.  F, F_out [L,B,h_kv,capacity].
 */
gkv_status gkv_pool_scores(gkv_ctx* ctx, const float* F, const int32_t* d_state, int32_t step,
                           int32_t kernel, float* F_out, void* stream);

/*
 * Eviction log (paper, Section 5: the positions of the tokens actually evicted during
 * generation are recorded and later build the sparse attention mask).  Call after
 * gkv_select_topk and BEFORE gkv_compact: writes, per unit, the original positions
 * (pos values) of the candidates that are not in keep_idx, ascending, padded with -1
 * to capacity - b entries (a compression from l rows drops l - b of them: s in steady
 * state, more when a prompt longer than the budget is compressed).
 * evicted [L,B,h_kv,capacity-b].  Sequences that are not compressed get all -1.
 */
gkv_status gkv_evicted_positions(gkv_ctx* ctx, const int32_t* keep_idx, const int32_t* pos,
                                 const int32_t* d_state, int32_t step, int32_t* evicted, void* stream);

/* The four compression calls above in order, on caller-provided S, F, keep_idx. */
gkv_status gkv_evict(gkv_ctx* ctx, const void* qwin, void* K, void* V, float* F_hist, int32_t* pos,
                     int32_t* d_state, int32_t step, int32_t len_max_host,
                     float* S, float* F, int32_t* keep_idx, void* workspace, void* stream);

/*
 * gkv_evict for callers that cannot allocate device memory and have no buffers to spare for the
 * intermediates: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same compression, same results in K, V, F_hist, pos and d_state; the local score,
 * the global score and the kept indices live in a fixed array of GKV_STATIC_SCRATCH_BYTES bytes
 * that is part of the library's device image (every GPU the library runs on holds it until the
 * process ends).  The call allocates and frees nothing (as long as the benchmark timing hooks of
 * gkv_bench.h are off, which they are unless switched on).  It needs
 *   2 * align256(4 * L*B*h_kv * capacity) + align256(4 * L*B*h_kv * (b - w))
 * bytes and returns GKV_ERR_SCRATCH, enqueuing nothing, if that exceeds the array (the 28-layer,
 * batch-8, b = 512 shape needs 6.4 MB).  The device of `stream` must be the current device.
 * Nothing in the array has to start at zero: every value read was written earlier in the same
 * call.  All calls on one GPU share the array, whatever context or stream they use, so two calls
 * that may overlap in time on one GPU race; serialise them (one stream, or events).
 */
#define GKV_STATIC_SCRATCH_BYTES (16u << 20)
gkv_status gkv_evict_static(gkv_ctx* ctx, const void* qwin, void* K, void* V, float* F_hist, int32_t* pos,
                            int32_t* d_state, int32_t step, int32_t len_max_host,
                            void* workspace, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GKV_H */

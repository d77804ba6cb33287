/*
 * lrqk.h — C ABI of the LRQK decode-step hot path for AMD MI355X (gfx950).
 *
 * LRQK ("Low Rank Query and Key" attention) keeps, per head, a rank-r key
 * factor A_K (l x r) on the GPU and the full-precision K/V rows in host
 * memory.  One decode step (Alg. 2, steps "proxy attention", "fetch missing",
 * "merge", followed by Attention(q, K_Omega, V_Omega) of Sec. 4.3) is:
 *
 *   a1  proxy scores   s = A_K q_hat^T                     (Alg. 2, top-k line)
 *   a2  selection      Omega_k = top(s, k) over [0, l-w),  Omega_l = [l-w, l)
 *                                                          (Sec. 4.1 "active" / "lite" tokens)
 *   a3  hit/miss       which of Omega_k already sit in the GPU cache, and where
 *                      the missing ones go                 (Sec. 4.1 hit-and-miss cache)
 *   a4  fetch          copy only the missing K/V rows host -> GPU cache
 *                                                          (Alg. 2 "Fetch missing", "merge")
 *   a5  attention      exact softmax attention of q over the k+w selected rows
 *                                                          (Sec. 4.3, last sentence)
 *
 * Conventions
 *   - Notation follows the paper: l context length, d head dimension, r rank,
 *     k active (top-k) tokens, w lite (recent) tokens.  B batch, Hq query heads,
 *     Hkv key/value heads, G = Hq/Hkv query heads per KV head, C cache slots
 *     per (batch, query head).
 *   - A_K, K, V and the lite rows are stored per (batch, KV head) and shared by
 *     the G query heads of the group; scores, selection, cache state, cache
 *     rows and outputs are per (batch, query head).  Query head h uses KV head
 *     h / G.
 *   - All arrays are dense, row-major, last index fastest, no padding.
 *   - "device" pointers are HIP device memory on the current device; "host"
 *     pointers are ordinary process memory; "pinned" is host memory allocated
 *     with hipHostMalloc (page-locked, device-visible).
 *   - Every buffer is allocated and owned by the caller.  The library keeps no
 *     pointer after a call returns, except inside an lrqk_plan.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Unless stated otherwise a call only enqueues work and returns.
 *   - Every entry point returns an int status: LRQK_OK (0) or a negative
 *     lrqk_status.  Arguments are validated on the host before anything is
 *     enqueued; on a validation error nothing is written.
 *   - Device pointers must be 16-byte aligned.
 */
#ifndef LRQK_H
#define LRQK_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LRQK_VERSION 200 /* major*10000 + minor*100 + patch */

typedef enum lrqk_status {
  LRQK_OK = 0,
  LRQK_EINVAL = -1, /* null or misaligned pointer, bad enum value, bad handle   */
  LRQK_ESHAPE = -2, /* sizes inconsistent or outside the supported range         */
  LRQK_EHIP = -3,   /* a HIP runtime call failed; see lrqk_last_hip_error()      */
  LRQK_ENOMEM = -4, /* workspace too small, or an allocation in plan_create failed */
  LRQK_ESTATE = -5  /* the cache state handed in is unusable (see lrqk_fetch_misses)   */
} lrqk_status;

enum { LRQK_KV_BF16 = 0, LRQK_KV_F32 = 1 };

/* How lrqk_decode_step / lrqk_fetch_misses move missing rows (step a4). */
enum {
  LRQK_FETCH_STAGED = 0, /* miss list -> host, host gathers rows into a pinned staging
                            buffer, one hipMemcpyAsync on the plan's side stream, then a
                            scatter kernel into the cache slots                        */
  LRQK_FETCH_DIRECT = 1, /* the GPU reads the rows straight out of the pinned host store
                            (device-visible host memory) and writes the cache slots; no host
                            synchronisation.  lrqk_fetch_misses does it in a kernel of its
                            own; lrqk_decode_step does it inside the attention kernel, so the
                            host-link reads overlap the HBM reads of the rows that hit      */
  LRQK_FETCH_GROUP = 2   /* as DIRECT, with the host link shared inside a KV group: K and V
                            exist once per KV head (Sec. 4, preliminaries), so a position that
                            several query heads of a group miss in the same step is one host
                            row; it is read once and written into the slot of each of those
                            heads.  The caches end up exactly as with the other modes; fewer
                            rows cross the link when the heads of a group want the same
                            tokens.  lrqk_decode_step: the shared fetch runs in one launch
                            with the attention over the rows that hit, the fetched rows are
                            attended by a second launch                                     */
};
/* May be OR-ed into the `mode` of lrqk_decode_step: estimate the candidate thresholds of the
 * selection from a sample of this step's proxy scores even though the layer carries thresholds
 * from its previous step (lrqk_layer.sel_thr).  For the first decode step of a sequence and
 * after anything that changes the score distribution wholesale.  Results never depend on it,
 * only speed does. */
#define LRQK_SELECT_FRESH 0x100

/*
 * Problem sizes of one layer's decode step.
 *   d        head dimension; only 128 is supported.
 *   r        rank of the factors, 4 <= r <= 128, multiple of 4.
 *   k        active tokens picked by proxy score, 1 <= k <= l - w, k <= 4096.
 *   w        lite tokens = the last w positions, always attended, 0 <= w <= 1024.
 *   C        cache slots per (batch, query head), k <= C <= 8192.
 *   kv_dtype element type of K/V rows (host store, cache, lite rows).
 *   scale    softmax scale applied to q.k (the usual 1/sqrt(d)).
 *   l_cap    rows allocated per head in the arrays that grow with the context (A_K, K_host,
 *            V_host, slot_of): their row stride.  0 means l (no room to grow); otherwise
 *            l <= l_cap < 2^24.  Where this header writes [.., l, ..] for one of those four
 *            arrays, read [.., l_cap, ..] with the first l rows in use.
 * Requirements: B >= 1, Hkv >= 1, Hq a multiple of Hkv, Hq/Hkv <= 8, l >= 1, l < 2^24.
 */
typedef struct lrqk_shape {
  int32_t B, Hq, Hkv, d, l, r, k, w, C;
  int32_t kv_dtype;
  float scale;
  int32_t l_cap;
} lrqk_shape;

/* Which call a workspace is sized for (lrqk_workspace_bytes). */
enum { LRQK_WS_SELECT = 1, LRQK_WS_ATTEND = 2, LRQK_WS_UPDATE = 3, LRQK_WS_PREFILL = 4 };

int lrqk_version(void);
const char* lrqk_status_string(int status);
/* Raw hipError_t of the most recent failing HIP call made by this library in
 * the calling thread (0 if none). */
int lrqk_last_hip_error(void);

/* Host-only check of a shape against the limits above. LRQK_OK / LRQK_EINVAL / LRQK_ESHAPE. */
int lrqk_validate_shape(const lrqk_shape* shape);

/* Bytes of device workspace the given call needs for this shape (0 on a bad
 * shape or selector).  Workspace contents need no initialisation. */
size_t lrqk_workspace_bytes(const lrqk_shape* shape, int which);

/*
 * a1 — proxy attention scores (Alg. 2, "compute proxy attention"; abstract: O(lr) per step).
 *   scores[b,h,i] = sum_{j<r} A_K[b, h/G, i, j] * q_hat[b, h, j],   i in [0, l)
 * accumulated in fp32 as one fused-multiply-add chain, j ascending, starting
 * from 0.0f, so the result is reproducible bit for bit.
 *   A_K     device, fp32 [B, Hkv, l, r]   read
 *   q_hat   device, fp32 [B, Hq, r]       read
 *   scores  device, fp32 [B, Hq, l]       written
 */
int lrqk_proxy_scores(const lrqk_shape* shape, const float* A_K, const float* q_hat,
                      float* scores, void* stream);

/*
 * a2 — active-token selection (Alg. 2, top(., k); Sec. 4.1: active + lite tokens).
 * For every (b,h): the k positions in [0, l-w) with the largest score; equal
 * scores are ordered by lower position first (-0.0f and +0.0f compare equal;
 * NaN scores are not supported).  Written in ascending position order.  The
 * lite set [l-w, l) is implicit and never listed.
 *   scores     device, fp32 [B, Hq, l]   read
 *   sel_idx    device, int32 [B, Hq, k]  written
 *   workspace  device, >= lrqk_workspace_bytes(shape, LRQK_WS_SELECT) bytes, 256-byte aligned
 * LRQK_ENOMEM if ws_bytes is too small.
 */
int lrqk_select_topk(const lrqk_shape* shape, const float* scores, int32_t* sel_idx,
                     void* workspace, size_t ws_bytes, void* stream);

/*
 * Cache state of one layer (all device memory):
 *   slot_of   int32 [B, Hq, l]  slot holding token i, or -1 if i is not on the GPU
 *   token_of  int32 [B, Hq, C]  token held by a slot, or -1 if the slot is empty
 *   last_used int32 [B, Hq, C]  step at which the slot's token was last selected, -1 if empty
 * slot_of and token_of are mutually inverse on the resident set.
 * lrqk_cache_init sets all three to -1 (an empty cache).
 */
int lrqk_cache_init(const lrqk_shape* shape, int32_t* slot_of, int32_t* token_of,
                    int32_t* last_used, void* stream);

/*
 * a3 — hit/miss resolution (Sec. 4.1: only tokens missing from the GPU cache are
 * fetched; Sec. 5.3 defines the miss rate as fetched rows / selected rows).
 * The paper's cache holds exactly the k active tokens; with C >= k slots a
 * replacement rule is needed and this library uses least-recently-selected:
 *   for each selected token, ascending position: resident -> hit, its slot's
 *   last_used becomes `step`; otherwise miss.  Victim slots are the slots whose
 *   last_used != step, ordered by (last_used ascending, slot ascending); the
 *   j-th miss (ascending position) takes the j-th victim; the evicted token's
 *   slot_of becomes -1; token_of / slot_of / last_used are updated.
 * With C == k this is the paper's behaviour (the cache ends up holding Omega_k).
 *   sel_idx   device int32 [B,Hq,k]  read; ascending, distinct, in [0, l-w)
 *   step      >= 0 and larger than every last_used currently stored
 *   slot_of, token_of, last_used     read and updated in place
 *   sel_slot  device int32 [B,Hq,k]  written: slot of sel_idx[..j] after the step
 *   hit       device uint8 [B,Hq,k]  written: 1 hit, 0 miss
 *   miss_tok, miss_slot device int32 [B,Hq,k]  written: first n_miss entries = the
 *             missing tokens (ascending) and the slots they were given; rest untouched
 *   n_miss    device int32 [B,Hq]    written
 * A head whose input breaks the contract (a position outside [0,l), or too
 * few victims because `step` was reused) does not fault: the offending entries
 * get sel_slot = -1 and that head's n_miss is written as -1.
 */
int lrqk_cache_resolve(const lrqk_shape* shape, const int32_t* sel_idx, int32_t step,
                       int32_t* slot_of, int32_t* token_of, int32_t* last_used,
                       int32_t* sel_slot, uint8_t* hit, int32_t* miss_tok, int32_t* miss_slot,
                       int32_t* n_miss, void* stream);

/*
 * a5 — exact attention over the selected rows (Sec. 4.3: Attention(q_t, K_Omega, V_Omega)
 * with the original q, K, V).
 *   out[b,h,:] = sum_{i in Omega} p_i V_i,  p = softmax_i(scale * q[b,h,:] . K_i)
 * Omega = the k cache rows named by sel_slot plus the w lite rows.  fp32
 * accumulation, max-subtracted softmax.  Entries of sel_slot outside [0, C)
 * are skipped.
 *   q                device fp32 [B,Hq,d]
 *   cacheK, cacheV   device kv_dtype [B,Hq,C,d]
 *   sel_slot         device int32 [B,Hq,k]
 *   liteK, liteV     device kv_dtype [B,Hkv,w,d]: the rows of positions l-w .. l-1, kept as a
 *                    ring: row j holds the position p of [l-w, l) with p mod w == j (the
 *                    attention does not depend on their order; may be NULL when w == 0)
 *   out              device fp32 [B,Hq,d]   written
 *   workspace        device, >= lrqk_workspace_bytes(shape, LRQK_WS_ATTEND), 256-byte aligned
 */
int lrqk_sparse_attend(const lrqk_shape* shape, const float* q, const void* cacheK,
                       const void* cacheV, const int32_t* sel_slot, const void* liteK,
                       const void* liteV, float* out, void* workspace, size_t ws_bytes,
                       void* stream);

/*
 * a5 for callers that cannot allocate: code under HIP graph capture, tight serving loops and
 * harnesses that forbid hipMalloc, which have no workspace to hand over either.  Same
 * arguments, kernels and results as lrqk_sparse_attend, without `workspace`: the partial
 * softmax states sit in a fixed array of LRQK_NOALLOC_SCRATCH_BYTES of device memory inside
 * the library (one copy per GPU, held until the process ends).  The call allocates and frees
 * nothing, on the host side of HIP or the device.
 *   LRQK_ENOMEM if lrqk_workspace_bytes(shape, LRQK_WS_ATTEND) exceeds the array (nothing is
 *   enqueued).  At the headline shape (32 heads, k = 2048, w = 64) the call needs 1.2 MB.
 * Every call on a GPU uses that GPU's one array: two calls whose work overlaps on the same
 * GPU (different streams, or threads) race.  Calls on one stream are ordered and safe.
 */
#define LRQK_NOALLOC_SCRATCH_BYTES (4u << 20)
int lrqk_sparse_attend_noalloc(const lrqk_shape* shape, const float* q, const void* cacheK,
                               const void* cacheV, const int32_t* sel_slot, const void* liteK,
                               const void* liteV, float* out, void* stream);

/*
 * A plan owns what the fused step and the fetch leg need beyond the caller's
 * buffers: device workspace, a side stream with events, and pinned staging
 * memory sized for `max_shape` (every later call must use a shape whose
 * B*Hq, l, k, w, C do not exceed it).  Created on the current device.
 */
typedef struct lrqk_plan lrqk_plan;
int lrqk_plan_create(const lrqk_shape* max_shape, lrqk_plan** plan_out);
int lrqk_plan_destroy(lrqk_plan* plan);

/*
 * a4 — fetch the missing rows (Alg. 2: "Fetch missing k_i, v_i from CPU K, V", "merge").
 * For every (b,h) and j < n_miss[b,h]:
 *   cacheK[b,h,miss_slot[b,h,j],:] = K_host[b,h/G,miss_tok[b,h,j],:]   (same for V), a bit copy.
 *   K_host, V_host  pinned host memory, kv_dtype [B,Hkv,l,d]
 *   miss_tok, miss_slot, n_miss  device, as written by lrqk_cache_resolve
 *   mode  LRQK_FETCH_STAGED: synchronises `stream` once to read the miss list on the
 *         host, then copies on the plan's side stream and makes `stream` wait for it.
 *         LRQK_FETCH_DIRECT, LRQK_FETCH_GROUP: one kernel on `stream`, no host
 *         synchronisation (GROUP needs the miss lists ascending, as lrqk_cache_resolve and
 *         lrqk_decode_step write them).
 *   total_miss_out  host int64*, optional: total rows fetched (STAGED only; the others write -1).
 * A head with n_miss < 0 (lrqk_cache_resolve could not place its misses): STAGED returns
 * LRQK_ESTATE after the synchronisation, with nothing copied; DIRECT and GROUP, which never see
 * the lists on the host, skip that head (its n_miss stays the only report).
 */
int lrqk_fetch_misses(lrqk_plan* plan, const lrqk_shape* shape, const void* K_host,
                      const void* V_host, const int32_t* miss_tok, const int32_t* miss_slot,
                      const int32_t* n_miss, void* cacheK, void* cacheV, int mode,
                      int64_t* total_miss_out, void* stream);

/* Buffers of one layer for the fused step. Device unless marked pinned. */
typedef struct lrqk_layer {
  float* A_K;          /* fp32 [B,Hkv,l,r]                       (written only by lrqk_append_token) */
  void* K_host;        /* pinned, kv_dtype [B,Hkv,l,d]           (likewise) */
  void* V_host;        /* pinned, kv_dtype [B,Hkv,l,d]           (likewise) */
  void* liteK;         /* kv_dtype [B,Hkv,w,d], ring of the last w rows (likewise) */
  void* liteV;         /* kv_dtype [B,Hkv,w,d]                   (likewise) */
  int32_t* slot_of;    /* int32 [B,Hq,l]  in/out */
  int32_t* token_of;   /* int32 [B,Hq,C]  in/out */
  int32_t* last_used;  /* int32 [B,Hq,C]  in/out */
  void* cacheK;        /* kv_dtype [B,Hq,C,d] in/out */
  void* cacheV;        /* kv_dtype [B,Hq,C,d] in/out */
  float* sel_thr;      /* fp32 [B,Hq] in/out, or NULL: candidate threshold of the selection
                          carried from one step of this layer to the next (see lrqk_decode_step);
                          set up with lrqk_select_state_init.  Only lrqk_decode_step uses it */
} lrqk_layer;

/*
 * Marks the carried selection thresholds of a layer as unknown (every entry NaN).
 *   sel_thr  device fp32 [B,Hq]  written
 */
int lrqk_select_state_init(const lrqk_shape* shape, float* sel_thr, void* stream);

/* Optional device outputs of the fused step (any may be NULL): the integer
 * results of a2/a3, bit-identical to what the separate calls produce. */
typedef struct lrqk_step_debug {
  int32_t* sel_idx;   /* [B,Hq,k] */
  int32_t* sel_slot;  /* [B,Hq,k] */
  uint8_t* hit;       /* [B,Hq,k] */
  int32_t* miss_tok;  /* [B,Hq,k] */
  int32_t* miss_slot; /* [B,Hq,k] */
  int32_t* n_miss;    /* [B,Hq]   */
  int32_t* link_rows; /* [B,Hkv]  LRQK_FETCH_GROUP only: rows read from the host store per KV
                         head = size of the union of its group's miss lists (cleared and
                         counted only when this pointer is given) */
} lrqk_step_debug;

/*
 * a1..a5 as one call (Alg. 2 from the proxy-attention line to the attention of
 * Sec. 4.3; Fig. 2: selection, then a small cache load overlapped with attention).
 * Scores never leave the library's workspace (for the shapes the filtered proxy-score
 * pass supports they are not even materialised).  STAGED: attention over the hit rows and
 * the lite rows runs on `stream` while the missing rows travel on the plan's side stream
 * and are attended afterwards; partial results are merged.  DIRECT: one attention launch
 * over all rows, the missing ones read from the host store and written to their slots on
 * the way.
 * Selection (shapes the filtered proxy-score pass supports): the pass over A_K keeps only the
 * positions whose score reaches a per-head candidate threshold, and the selection is made
 * exactly among those; a head whose candidates turn out unusable (fewer than k) is redone
 * exactly from all its scores, so the threshold affects speed, never the result.  The
 * threshold is estimated from a sample of this step's scores (two small launches) when
 * layer->sel_thr is NULL or `mode` carries LRQK_SELECT_FRESH; otherwise it is
 * layer->sel_thr[b,h] * |q_hat[b,h]|, the value the previous step's selection left there (the
 * score at rank 1.5 k, per unit of |q_hat|), and every step rewrites sel_thr for the next one.
 * An entry that is NaN (lrqk_select_state_init) sends its head down the exact, slow route.
 *   q_hat  device fp32 [B,Hq,r];  q  device fp32 [B,Hq,d];  out  device fp32 [B,Hq,d]
 *   step   as in lrqk_cache_resolve
 *   mode   LRQK_FETCH_STAGED (one host synchronisation per call, to read the miss
 *          list), LRQK_FETCH_DIRECT or LRQK_FETCH_GROUP (fully asynchronous), optionally
 *          | LRQK_SELECT_FRESH
 *   dbg    optional
 *   total_miss_out  host int64*, optional (STAGED: rows fetched; DIRECT, GROUP: -1)
 */
int lrqk_decode_step(lrqk_plan* plan, const lrqk_shape* shape, int32_t step,
                     const lrqk_layer* layer, const float* q_hat, const float* q, float* out,
                     int mode, const lrqk_step_debug* dbg, int64_t* total_miss_out,
                     void* stream);

/*
 * u1 — decode-time update of the factors (Alg. 2, from the initial guess of k_hat to the two
 * gradient steps on B_Q and B_K; Sec. 4.2 decode objective and update rules; App. A.2 step
 * lengths).  Runs BEFORE the step's proxy scores: it produces the q_hat that lrqk_proxy_scores
 * / lrqk_decode_step take, and the k_hat that lrqk_append_token adds to A_K.
 * For the new projections q_t (per query head) and k_t (per KV head):
 *   k_hat <- k B_K^T (B_K B_K^T)^-1                                   (lambda_d1 = 0 guess)
 *   n_iter times:
 *     q_hat <- m_lq M_rq^-1 for every query head, with
 *        m_lq = q B_Q^T + lambda_d1 (q.k) k_hat + lambda_d2 (q K_Om^T) A_Om
 *        M_rq = B_Q B_Q^T + lambda_d1 k_hat^T k_hat + lambda_d2 A_Om^T A_Om
 *     k_hat <- (k B_K^T + lambda_d1 sum_g (q_g.k) q_hat_g)
 *              (B_K B_K^T + lambda_d1 sum_g q_hat_g^T q_hat_g)^-1     (sums over the G query
 *              heads that share the KV head; G = 1 gives the paper's rule)
 *   B_Q <- B_Q - eta_Q q_hat^T (q_hat B_Q - q),  B_K <- B_K - eta_K k_hat^T (k_hat B_K - k),
 *   each eta the exact minimiser along its gradient; a zero gradient leaves B unchanged.
 * Omega = the rows attended at the previous step: the previous selection (A_K rows at
 * sel_idx_prev, K rows in the cache slots sel_slot_prev) and the lite window [l-w, l) (A_K
 * rows l-w .. l-1, K rows in layer->liteK); q K_Om^T is the raw dot product.  Entries of the
 * previous selection with a position outside [0, l) or a slot outside [0, C) are left out.
 * The loop runs exactly n_iter rounds (the paper uses at most 2); there is no tolerance test.
 * All arithmetic is fp32 (App. B.1).  Supported ranks: r in {8, 16, 32, 64}.
 *   layer          A_K, cacheK and liteK are read (device)
 *   sel_idx_prev, sel_slot_prev  device int32 [B,Hq,k], as written by the previous step
 *   q              device fp32 [B,Hq,d]
 *   k_new          device kv_dtype [B,Hkv,d]
 *   B_Q            device fp32 [B,Hq,r,d]   updated in place
 *   B_K            device fp32 [B,Hkv,r,d]  updated in place
 *   lambda_d1, lambda_d2  >= 0, finite;  1 <= n_iter <= 64
 *   q_hat          device fp32 [B,Hq,r]   written
 *   k_hat          device fp32 [B,Hkv,r]  written
 *   workspace      device, >= lrqk_workspace_bytes(shape, LRQK_WS_UPDATE), 256-byte aligned
 * LRQK_ESHAPE for an unsupported rank, LRQK_ENOMEM if ws_bytes is too small.
 */
int lrqk_factor_update(const lrqk_shape* shape, const lrqk_layer* layer,
                       const int32_t* sel_idx_prev, const int32_t* sel_slot_prev, const float* q,
                       const void* k_new, float* B_Q, float* B_K, float lambda_d1,
                       float lambda_d2, int32_t n_iter, float* q_hat, float* k_hat,
                       void* workspace, size_t ws_bytes, void* stream);

/*
 * u2 — the new token joins the context (Alg. 2: A_K <- [A_K; k_hat_t], K_Omega <- [K'; k_t],
 * V_Omega <- [V'; v_t], "Async k_t, v_t to CPU").  With l = shape->l the current length:
 *   A_K[b,kv,l,:] = k_hat[b,kv,:];  K_host[b,kv,l,:] = k_new[b,kv,:];  V_host likewise (bit
 *   copies, written by the GPU into the pinned store: asynchronous to the host, complete
 *   when the work enqueued on `stream` has finished);  the lite ring row l mod w (which held
 *   position l - w) receives k_new / v_new;  slot_of[b,h,l] = -1.
 * Afterwards the context has l + 1 rows: the caller passes shape->l + 1 to the following
 * calls (the new token is then inside the lite window [l+1-w, l+1), always attended).
 * Needs room for the row: shape->l_cap > shape->l, else LRQK_ESHAPE.
 *   layer   A_K, K_host, V_host, liteK, liteV, slot_of are written as described
 *   k_hat   device fp32 [B,Hkv,r]      (from lrqk_factor_update)
 *   k_new, v_new  device kv_dtype [B,Hkv,d]
 */
int lrqk_append_token(const lrqk_shape* shape, const lrqk_layer* layer, const float* k_hat,
                      const void* k_new, const void* v_new, void* stream);

/*
 * p1 — prefill factorisation (Alg. 1; Sec. 4.1 "Prefill": Q K^T ~ A_Q A_K^T with Q ~ A_Q B_Q,
 * K ~ A_K B_K, solved by alternating closed-form updates; App. A.1).  Produces the A_K that
 * the decode step scans and the B_Q, B_K that lrqk_factor_update continues from.
 * Starting from the A_Q, A_K handed in (the paper draws them from N(0,1); the caller draws),
 * n_iter rounds of
 *   B_Q <- (A_Q^T A_Q)^-1 A_Q^T Q                                  per query head
 *   B_K <- (A_K^T A_K)^-1 A_K^T K                                  per KV head
 *   A_K <- K (sum_g Q_g^T A_Q,g + lambda_pK B_K^T)
 *            (sum_g A_Q,g^T A_Q,g + lambda_pK B_K B_K^T)^-1        per KV head, sums over the
 *                                                                  G query heads of its group
 *   A_Q <- Q (K^T A_K + lambda_pQ B_Q^T)(A_K^T A_K + lambda_pQ B_Q B_Q^T)^-1   per query head
 * in this order (G = 1 gives the paper's rules).  B_Q, B_K are those computed at the top of
 * the last round.  Exactly n_iter rounds (the paper uses at most 2); no convergence test.
 * fp32 arithmetic on the matrix cores (App. B.1).  Supported ranks: r in {8, 16, 32, 64}.
 * Of `shape`, B, Hq, Hkv, d, l, r, kv_dtype and l_cap are used.
 *   Q     device kv_dtype [B,Hq,l,d]     read
 *   K     device kv_dtype [B,Hkv,l,d]    read
 *   A_Q   device fp32 [B,Hq,l,r]         in: initial values, out: result
 *   A_K   device fp32 [B,Hkv,l_cap,r]    in: initial values, out: result (rows >= l untouched)
 *   B_Q   device fp32 [B,Hq,r,d]         written
 *   B_K   device fp32 [B,Hkv,r,d]        written
 *   lambda_pQ, lambda_pK  >= 0, finite;  1 <= n_iter <= 64
 *   workspace  device, >= lrqk_workspace_bytes(shape, LRQK_WS_PREFILL), 256-byte aligned
 * A_Q^T A_Q and A_K^T A_K must be positive definite (they are for generic inputs with l >= r).
 */
int lrqk_prefill_factorize(const lrqk_shape* shape, const void* Q, const void* K, float* A_Q,
                           float* A_K, float* B_Q, float* B_K, float lambda_pQ, float lambda_pK,
                           int32_t n_iter, void* workspace, size_t ws_bytes, void* stream);

/*
 * Instrumentation (not part of the method): GPU time of the kernels of lrqk_decode_step, each
 * taken from a pair of HIP events attached to the kernel itself (they hold its own start and
 * end, so neither the gaps between launches nor the events' own cost are included).
 * lrqk_plan_profile(plan, n) arms the next n calls of lrqk_decode_step on this plan (n = 0
 * switches it off); lrqk_plan_profile_read waits for the recorded steps, adds up every
 * slot's kernel time into ms_sum[LRQK_PROFILE_SLOTS] (milliseconds, summed over the steps;
 * 0 for kernels the steps did not launch) and re-arms.  Slots:
 */
enum {
  LRQK_SLOT_SAMPLE = 0,      /* threshold estimate: scores of the sampled rows          */
  LRQK_SLOT_THRESHOLD = 1,   /* threshold estimate: histogram of the samples            */
  LRQK_SLOT_PROXY = 2,       /* a1, the pass over A_K                                   */
  LRQK_SLOT_SELECT = 3,      /* a2 (+ a3 where one kernel does both; of the multi-launch
                                selection of very long contexts only the first kernel)  */
  LRQK_SLOT_RESOLVE = 4,     /* a3 as a kernel of its own                               */
  LRQK_SLOT_FETCH = 5,       /* STAGED: scatter of the copied rows into the cache slots */
  LRQK_SLOT_ATTEND = 6,      /* a5 partials (DIRECT: with the fetch; STAGED: hit rows)  */
  LRQK_SLOT_ATTEND_MISS = 7, /* STAGED: a5 partials over the rows that were fetched     */
  LRQK_SLOT_COMBINE = 8,     /* a5 merge of the partials                                */
  LRQK_PROFILE_SLOTS = 9
};
int lrqk_plan_profile(lrqk_plan* plan, int n_steps);
int lrqk_plan_profile_read(lrqk_plan* plan, double* ms_sum, int* n_steps_out);

/*
 * Instrumentation: time the dominant kernel alone.  Runs step a1's pass over A_K exactly as
 * lrqk_decode_step launches it for this shape (the filtered proxy-score kernel, its thresholds
 * taken from sel_thr [B,Hq] as in a step that carries them (device, a layer's array after a
 * step with this kind of q_hat), or, with sel_thr NULL, estimated once from a sample for q_hat;
 * the plain proxy-score kernel for shapes that do not use the filter), n_launches times back
 * to back on `stream`, cycling through the n_list
 * device arrays A_K_list[i] (each [B,Hkv,l,r] fp32, e.g. one per layer, so that no cache
 * holds them), bracketed by two HIP events: microseconds per launch, gaps between launches
 * included.  For the filtered kernel a second series of at most 64 launches attaches a pair
 * of events to every kernel (they hold that kernel's own start and end); the average of
 * those durations is reported instead when it is positive and not above the bracketed
 * figure.  Synchronises; *avg_us_out = microseconds per launch.  Results go to the plan's
 * workspace and are discarded.
 */
int lrqk_plan_time_proxy_pass(lrqk_plan* plan, const lrqk_shape* shape,
                              const float* const* A_K_list, int n_list, const float* q_hat,
                              const float* sel_thr, int n_launches, float* avg_us_out,
                              void* stream);

/*
 * Instrumentation: copy `bytes` (a multiple of 16) from src to dst, both device memory,
 * 16-byte aligned, with a plain one-load-one-store kernel.  Its HBM traffic is known
 * (bytes read + bytes written), which calibrates the hardware byte counters that the
 * measured traffic of the other kernels is scaled by.
 */
int lrqk_calib_copy(void* dst, const void* src, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LRQK_H */

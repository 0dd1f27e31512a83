/*
 * purekv.h -- C ABI of the PureKV hot path for AMD MI355X (gfx950).
 *
 * The library implements, on one GPU, the data-parallel part of PureKV:
 *   - ST-SpAttn prefill attention over F frames x P patches of video tokens followed by
 *     T text tokens (paper Sec. 3.2), and dense causal attention for the low layers (Eq. 1);
 *   - the recent-window column-sum importance C^low (Eq. 2);
 *   - the V-norm weighting S = C * ||V|| (Eq. 3 for the low layer, Eq. 4 for the high layers that
 *     reuse C^low with their own V) and the per-KV-head selection "recent w + top h" (Sec. 3.1);
 *   - the gather of the kept K/V rows into a compact cache;
 *   - single-token decode attention against that compact cache, alone or fused with the append of the token;
 *   - the layer stack that ties these together (which layers are dense, which estimate the importance);
 *   - two calibration loops that measure what the board sustains (no part of the method).
 *
 * Conventions
 *   - Token order: video tokens frame-major (index i < F*P: frame i / P, patch i % P), then text.
 *     N = F*P + T.  P = patch_h * patch_w; "the corresponding token of the previous frame" is i - P.
 *   - Q, K, V and O are bf16 tensors indexed (head, token, channel) with head_dim contiguous; the head and
 *     token strides are fields of purekv_shape_t (elements; 0 = packed [H, N, d]), so the same calls serve
 *     head-major tensors and the token-major [N, H * d] slices a decoder's QKV projection emits:
 *       Q (Hq, N, d), K and V (Hkv, N, d), O (Hq, N, d).   Query head hq reads KV head hq / (Hq/Hkv).
 *     K and V share one pair of strides.  Everything the library itself produces for its own later use
 *     (log-sum-exp, column sums, scores, kept indices, the compact cache) is packed.
 *   - Every data pointer is a DEVICE pointer owned by the caller (16-byte aligned), unless the
 *     argument is documented as a host pointer.  `stream` is a hipStream_t passed as void* (NULL = default
 *     stream).  Calls enqueue work on `stream` and return; they do not synchronise and, except for plan
 *     creation/destruction, do not allocate.  The caller keeps buffers alive until the stream has run.
 *   - Return value: PUREKV_OK (0) or a negative purekv_status.  All argument validation happens on the
 *     host before any GPU call, so EINVAL / EUNSUPPORTED / EWORKSPACE never leave work half enqueued.
 *   - Workspaces: purekv_workspace_bytes() gives the size an operation needs; pass a device buffer of at
 *     least that size (may be NULL when the size is 0), 256-byte aligned.  The PREFILL and DECODE workspaces begin
 *     with arrival counters through which workgroups of one launch hand partial results to each other: such a
 *     buffer must be initialised ONCE with purekv_workspace_init before its first use (and again after a failed
 *     launch, or after anything else wrote to it); every call leaves it ready for the next.  Calls that may overlap
 *     on the GPU need workspaces of their own; a plan may be shared by any number of streams.
 */
#ifndef PUREKV_H_
#define PUREKV_H_

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define PUREKV_API __attribute__((visibility("default")))
#else
#define PUREKV_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  PUREKV_OK = 0,
  PUREKV_EINVAL = -1,        /* null pointer, non-positive size, inconsistent arguments          */
  PUREKV_EUNSUPPORTED = -2,  /* head_dim not in {64, 128}, unknown pattern bits                   */
  PUREKV_EWORKSPACE = -3,    /* workspace smaller than purekv_workspace_bytes() says              */
  PUREKV_EHIP = -4,          /* a HIP runtime call failed (no device, launch failure, ...)        */
  PUREKV_ENOMEM = -5         /* host allocation failed                                            */
} purekv_status;

/* Sparsity pattern bits (Sec. 3.2).  0 = dense causal attention (Eq. 1). */
#define PUREKV_PATTERN_DENSE 0u
#define PUREKV_PATTERN_SPATIAL 1u  /* keys of the first frame and of the query's own frame         */
#define PUREKV_PATTERN_TEMPORAL 2u /* keys of the first frame, the same patch one frame back, self */
#define PUREKV_PATTERN_ST 3u       /* union of both paths                                          */

typedef struct {
  int32_t n_frames, patch_h, patch_w, n_text; /* F >= 1, patch_h, patch_w >= 1, T >= 0            */
  int32_t n_q_heads, n_kv_heads, head_dim;    /* Hq % Hkv == 0; head_dim 64 or 128                */
  uint32_t pattern;                           /* PUREKV_PATTERN_*                                 */
  float softmax_scale;                        /* 0 => 1/sqrt(head_dim) (Eq. 1)                    */
  /* Element strides of the (head, token) axes of Q, of K and V, and of O; head_dim is always contiguous.
   * A pair of zeros means packed [H, N, d] (head stride N * d, token stride d); otherwise both must be given.
   * Requirements (else EINVAL): multiples of 8 elements (16-byte rows), token stride >= d and < 2^23, and the
   * byte span of each tensor below 2^31.  Overlapping (head, token) rows are the caller's business for the
   * inputs and undefined for O. */
  int64_t q_stride_head, q_stride_tok;
  int64_t kv_stride_head, kv_stride_tok;
  int64_t o_stride_head, o_stride_tok;
} purekv_shape_t;

typedef struct purekv_plan purekv_plan_t;

typedef enum {
  PUREKV_OP_PREFILL = 0,
  PUREKV_OP_IMPORTANCE = 1,
  PUREKV_OP_TOPK = 2,
  PUREKV_OP_COMPACT = 3,
  PUREKV_OP_DECODE = 4
} purekv_op;

/*
 * Plan: the static block structure of the mask for one shape (Sec. 3.2: the pattern depends only on
 * F, P, T) and the static schedule of the prefill kernel.
 *
 * A prefill workgroup has PUREKV_WAVES wavefronts of PUREKV_BLOCK (32) query rows each.  The plan stacks
 * Gs query heads that share a KV head times R row blocks in one workgroup (wavefront w: row block w / Gs,
 * head w % Gs; Gs * R <= PUREKV_WAVES), because the mask depends on the row and not on the head: stacked
 * heads need exactly the same key tiles.  A query tile is R * 32 rows.  For every query tile the plan lists
 * the tiles of PUREKV_BK (64) keys that hold at least one allowed (query, key) pair and, per (row block rb,
 * 32-key half kb) of such a tile, a `need` bit (bit 2*rb + kb: the pair of blocks holds an allowed pair) and a
 * two-bit kind (bits 4*rb + 2*kb of `kinds`) that says how cheaply the element mask can be applied:
 * PUREKV_KIND_FULL (every pair allowed), _CAUSAL (allowed <=> key <= query), _PREV (allowed <=> key ==
 * query - P) or _GENERAL (the whole predicate).  Long lists are cut into slices (work items) whose partial
 * results are merged; every (work item, head group) unit is dealt to one of the persistent workgroups of the
 * prefill kernel (one per compute unit), longest first, KV heads kept on fixed XCDs where the head counts
 * allow it.
 *
 * purekv_plan_create builds the lists on the host and uploads them to the current device (KB to a few
 * MB, owned by the plan; `stream` orders the upload).  purekv_plan_create_host only builds the host
 * lists for `n_workgroups` persistent workgroups (no GPU needed; such a plan can be inspected but not
 * launched: compute calls return EINVAL).  `*out` is written only on success.  Destroy with
 * purekv_plan_destroy (NULL is accepted).
 */
#define PUREKV_BLOCK 32
#define PUREKV_BK 64
#define PUREKV_WAVES 8
#define PUREKV_KIND_FULL 0u
#define PUREKV_KIND_CAUSAL 1u
#define PUREKV_KIND_PREV 2u
#define PUREKV_KIND_GENERAL 3u
PUREKV_API int purekv_plan_create(const purekv_shape_t* shape, purekv_plan_t** out, void* stream);
PUREKV_API int purekv_plan_create_host(const purekv_shape_t* shape, int32_t n_workgroups, purekv_plan_t** out);
PUREKV_API int purekv_plan_destroy(purekv_plan_t* plan);
/*
 * Plans over a subset of the query heads, for models that give different heads different patterns (the other
 * reading of the "dual path" of Sec. 3.2: some heads spatial, others temporal): head_mask is a HOST array of
 * n_q_heads bytes, non-zero = the head belongs to this plan (at least one).  A prefill call with such a plan
 * computes the selected heads only and leaves the other heads' rows of `out` (and `lse`) untouched, so one call per
 * pattern, each with the plan of its heads, fills `out`.  A subset made of whole stacks of heads (e.g. whole KV groups)
 * keeps the stacked workgroup shape; any other subset is planned one head per workgroup.
 * The other entry points ignore the subset.
 */
PUREKV_API int purekv_plan_create_heads(const purekv_shape_t* shape, const uint8_t* head_mask, purekv_plan_t** out,
                                        void* stream);
PUREKV_API int purekv_plan_create_heads_host(const purekv_shape_t* shape, const uint8_t* head_mask, int32_t n_workgroups,
                                             purekv_plan_t** out);

/* Window plans, for the designated low layer (Sec. 3.1): Eq. 2 reads the attention probabilities of the last w
 * query rows only (the recent window), so only those rows' log-sum-exp is needed from the prefill.  On such a plan
 * a prefill call with `lse` given writes lse[h, i] for i >= N - w only and leaves every other element of `lse`
 * untouched, and only the workgroups that own those rows carry the exact row sum through their tile loop (it costs
 * the loop 7-10 %); everything else -- outputs, workspaces, every other call -- is as for purekv_plan_create.
 * purekv_lowlayer_importance on such a plan refuses a window larger than w (PUREKV_EINVAL).  1 <= w <= N, else
 * PUREKV_EINVAL. */
PUREKV_API int purekv_plan_create_window(const purekv_shape_t* shape, int32_t w, purekv_plan_t** out, void* stream);
PUREKV_API int purekv_plan_create_window_host(const purekv_shape_t* shape, int32_t w, int32_t n_workgroups,
                                              purekv_plan_t** out);

/* Plan inspection (host memory).  counts[0..15] = N, number of query tiles, number of work items,
 * number of (query tile, key tile) references, number of (row block, 32-key block) pairs computed per
 * query head, number of query tiles whose list is split, number of persistent workgroups, R (row blocks
 * per query tile), Gs (stacked heads), number of head groups (Hq / Gs), then the computed pairs by kind
 * (full, causal, prev, general), then the window w of a window plan (0 for any other plan) and the first persistent
 * workgroup of those that own the window's rows (0 when the plan is not divided). */
PUREKV_API int purekv_plan_counts(const purekv_plan_t* plan, int64_t counts[16]);
/* Copies the key-tile list of query tile `qt` into refs[0 .. 3*cap): triples {key tile index, need bits,
 * kind bits}.  Returns the list length (may exceed cap; then only cap triples are written) or a negative
 * status. */
PUREKV_API int purekv_plan_qtile_list(const purekv_plan_t* plan, int32_t qt, int32_t* refs, int32_t cap);
/* Copies work item `it` as {query tile, first list position, tile count, split index, number of
 * splits, partial-result slot or -1}.  Returns PUREKV_OK or a negative status. */
PUREKV_API int purekv_plan_item(const purekv_plan_t* plan, int32_t it, int32_t item[6]);
/* Copies the units of persistent workgroup `wg`, in execution order, into units[0 .. 2*cap): pairs {work
 * item, first query head of the group}.  Returns the number of units (may exceed cap) or a negative status. */
PUREKV_API int purekv_plan_queue(const purekv_plan_t* plan, int32_t wg, int32_t* units, int32_t cap);
/* Copies the steps of persistent workgroup `wg`, in execution order, into steps[0 .. 4*cap): one record of four
 * values per step: {byte offset of the key tile's first row in K and V, need bits | last << 16 | first << 17 |
 * (rows of the tile that exist - 1) << 18 | owner << 24, kind bits, first key of the tile}.  A step stages one key
 * tile of its unit's list (Sec. 3.2: the lists are the pattern's block indices); `first` / `last` mark the ends of a
 * unit, units follow each other in the order purekv_plan_queue reports; `owner` marks the one step of the launch
 * that also emits the squared norms of the tile's V rows.  Returns the number of steps (may exceed cap) or a
 * negative status. */
PUREKV_API int purekv_plan_steps(const purekv_plan_t* plan, int32_t wg, int32_t* steps, int32_t cap);

/* Spearman's rank correlation between two score arrays, row by row (Sec. 3.3, Eq. 5-7: the check that the scores
 * estimated with a low layer's column sums, Eq. 4, rank the non-recent keys like the scores of the layer's own
 * attention, Eq. 6).  rank(S) is a score's position in its row's descending order, equal scores in index order (the
 * tie rule of purekv_topk_select; -0.0 equals +0.0; NaN scores are unsupported), and
 *   rho = 1 - 6 sum_j (r_hat_j - r_j)^2 / (n (n^2 - 1)),   n = n_keys.
 *   s_hat, s: device fp32 [n_rows, n_keys] (packed rows; e.g. the s_out of two purekv_topk_select calls);
 *   sum_d2_out: device uint64 [n_rows], the sums of squared rank differences (exact); rho_out: device fp64 [n_rows]
 *   or NULL.  Needs no plan and no workspace; the work is quadratic in n_keys (a diagnostic, not a step of the path).
 *   2 <= n_keys <= 131072 (so that rho is the correctly rounded value of the exact quotient), n_rows >= 1, else
 *   PUREKV_EINVAL. */
PUREKV_API int purekv_spearman(const float* s_hat, const float* s, int32_t n_rows, int32_t n_keys, uint64_t* sum_d2_out,
                               double* rho_out, void* stream);

/* Device workspace bytes needed by `op` for this plan.  `n_layers`, `w` and `cap` are read by the ops
 * that take them (TOPK: n_layers, w; DECODE: cap); pass 0 otherwise.  What lives there: PREFILL, the partial
 * results of query tiles whose key list is cut into slices (the text rows of Sec. 3.2 see every key); TOPK, the
 * scores S of Eq. 3 / Eq. 4 when the caller does not ask for them; DECODE, the per-chunk partial results of the
 * decode stage.  IMPORTANCE (Eq. 2) and COMPACT need none. */
PUREKV_API size_t purekv_workspace_bytes(const purekv_plan_t* plan, int op, int32_t n_layers, int32_t w, int32_t cap);
/* Prepares a fresh workspace of `op` (same n_layers, w, cap as for purekv_workspace_bytes): clears the arrival
 * counters of a PREFILL or DECODE workspace with a small kernel on `stream` (no memset node: the call may be
 * captured in a graph); nothing to do for the other ops.  EWORKSPACE if ws is NULL or too small while the op needs
 * one. */
PUREKV_API int purekv_workspace_init(const purekv_plan_t* plan, int op, void* ws, size_t ws_bytes, int32_t n_layers,
                                     int32_t w, int32_t cap, void* stream);

/*
 * Prefill attention under the plan's pattern (Sec. 3.2; Eq. 1 when the pattern is dense):
 *   out[hq, i, :] = sum_j A[i, j] v[kv, j, :],  A = softmax over the allowed keys of q_i . k_j * scale.
 * The attention matrix is never stored.  bf16 inputs, bf16 MFMA products, fp32 accumulation and softmax.
 *   q (Hq, N, d), k, v (Hkv, N, d), out (Hq, N, d): bf16 device, laid out by the plan's strides.
 *   lse: optional fp32 device [Hq, N] (packed): natural-log sum of exponentials of every row's scaled logits
 *        (needed by purekv_lowlayer_importance); NULL to skip.
 */
PUREKV_API int purekv_st_spattn_prefill(const purekv_plan_t* plan, const void* q, const void* k, const void* v,
                             void* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * The same prefill that also emits, at no extra pass over V, what the V-norm weighting of Eq. 3 / Eq. 4 needs of this
 * layer's values: vnorm2[kv, j] = sum_c v[kv, j, c]^2 for every key (fp32 [Hkv, N], packed), computed from the V tiles
 * while they sit in on-chip memory for the second product (every key tile has one owner step in the plan's
 * schedule).  purekv_topk_select_vnorm then weighs C with these norms instead of streaming V again.  With a plan
 * over a head subset, rows of KV heads none of whose query heads belong to the plan are left untouched.
 */
PUREKV_API int purekv_st_spattn_prefill_vnorm(const purekv_plan_t* plan, const void* q, const void* k, const void* v,
                                              void* out, float* lse, float* vnorm2, void* ws, size_t ws_bytes,
                                              void* stream);

/*
 * Recent-window column sums (Eq. 2), summed over the query heads of each KV group:
 *   c_out[kv, j] = sum_{hq in group kv} sum_{i = N-w}^{N-1} exp(q_i . k_j * scale - lse[hq, i]),  0 <= j < N-w,
 * over the pairs (i, j) the plan's pattern allows.  `lse` is the one written by the prefill call of the
 * same layer with the same plan.  fp32 throughout after the bf16 products; summation order is fixed, so
 * results are reproducible bit for bit.
 *   q (Hq, N, d), k (Hkv, N, d) bf16 by the plan's strides; lse [Hq, N] fp32; c_out [Hkv, N-w] fp32.   1 <= w <= N.
 */
PUREKV_API int purekv_lowlayer_importance(const purekv_plan_t* plan, const void* q, const void* k, const float* lse,
                               int32_t w, float* c_out, void* ws, size_t ws_bytes, void* stream);

/*
 * V-norm weighting and selection (Eq. 3 / Eq. 4 and the selection rule of Sec. 3.1), for `n_layers`
 * layers that share one C:
 *   s[l, kv, j] = c[kv, j] * ||v[l, kv, j, :]||_2   (fp32; s = c when v is NULL, then n_layers must be 1),
 *   idx_out[l, kv, 0..h)   = the h indices j < N-w with the largest s, ties to the lower index, ascending,
 *   idx_out[l, kv, h..h+w) = N-w .. N-1.
 *   c [Hkv, N-w] fp32; v: bf16, layer l at v + l * v_layer_stride elements, each (Hkv, N, d) by the plan's K/V strides;
 *   idx_out [n_layers, Hkv, h+w] int32; s_out optional [n_layers, Hkv, N-w] fp32 (NULL to skip).
 *   1 <= w <= N, 0 <= h <= N-w.  Scores must not be NaN; -0.0 ranks equal to +0.0.
 */
PUREKV_API int purekv_topk_select(const purekv_plan_t* plan, const float* c, const void* v, int64_t v_layer_stride,
                       int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, float* s_out,
                       void* ws, size_t ws_bytes, void* stream);

/*
 * purekv_topk_select with the squared norms purekv_st_spattn_prefill_vnorm emitted instead of V (Eq. 3 / Eq. 4):
 *   s[l, kv, j] = c[kv, j] * sqrt(vnorm2[l, kv, j]),  vnorm2: fp32, layer l at + l * vn_layer_stride elements, each
 *   [Hkv, N]; everything else as for purekv_topk_select (the workspace holds the scores when s_out is NULL).
 */
PUREKV_API int purekv_topk_select_vnorm(const purekv_plan_t* plan, const float* c, const float* vnorm2,
                                        int64_t vn_layer_stride, int32_t n_layers, int32_t w, int32_t h,
                                        int32_t* idx_out, float* s_out, void* ws, size_t ws_bytes, void* stream);

/*
 * purekv_topk_select for callers that cannot allocate or hold a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same arguments and results as purekv_topk_select with
 * s_out == NULL, but the scores live in a buffer that is part of the library's device image (4 MiB per GPU, held
 * from library load until the process ends) instead of a caller workspace.  The call allocates nothing.
 *   Limit: n_layers * Hkv * (N - w) <= 2^20 scores, else PUREKV_EWORKSPACE (use purekv_topk_select).
 *   All calls on one GPU share that buffer: calls that may overlap on the GPU (different streams) race; calls on one
 *   stream are ordered and safe.  The plan must have been created on the device the call runs on.
 */
#define PUREKV_STATIC_SCORES_MAX (1 << 20)
PUREKV_API int purekv_topk_select_static(const purekv_plan_t* plan, const float* c, const void* v,
                                         int64_t v_layer_stride, int32_t n_layers, int32_t w, int32_t h,
                                         int32_t* idx_out, void* stream);

/*
 * Compaction: kc[l, kv, r, :] = k[l, kv, idx[l, kv, r], :] for r < n_keep, same for v (bit copy).
 *   k, v: bf16, layer l at + l * kv_layer_stride elements, each (Hkv, N, d) by the plan's K/V strides;
 *   idx [n_layers, Hkv, n_keep] int32 with values in [0, N) (not checked on the device beyond clamping);
 *   kc, vc [n_layers, Hkv, cap, d] bf16, cap >= n_keep; rows r >= n_keep are left untouched.
 */
PUREKV_API int purekv_kv_compact(const purekv_plan_t* plan, const void* k, const void* v, int64_t kv_layer_stride,
                      int32_t n_layers, const int32_t* idx, int32_t n_keep, void* kc, void* vc,
                      int32_t cap, void* stream);

/* Appends one token's k_new, v_new [Hkv, d] as row n_cached of kc, vc [Hkv, cap, d] (n_cached < cap): the cache
 * the decode stage of the paper's inference-speed table reads grows by the token it has just produced (Sec. 4.3;
 * the kept set of Sec. 3.1 plus every later token). */
PUREKV_API int purekv_kv_append(const purekv_plan_t* plan, const void* k_new, const void* v_new, void* kc, void* vc,
                     int32_t n_cached, int32_t cap, void* stream);

/*
 * Decode attention of one new token against the compact cache (the decode stage the paper times in its
 * inference-speed table):  out[hq, :] = softmax(q_new[hq] . kc[kv, 0..n_cached)^T * scale) vc[kv, 0..n_cached).
 *   q_new, out [Hq, d] bf16; kc, vc [Hkv, cap, d] bf16; 1 <= n_cached <= cap.
 */
PUREKV_API int purekv_decode_attn(const purekv_plan_t* plan, const void* q_new, const void* kc, const void* vc,
                       int32_t n_cached, int32_t cap, void* out, void* ws, size_t ws_bytes, void* stream);

/*
 * One decode step in one launch (the decode stage of the paper's inference-speed table, per generated token):
 * stores k_new, v_new [Hkv, d] as row n_cached of kc, vc (as purekv_kv_append does) and attends q_new over rows
 * 0 .. n_cached inclusive (as purekv_decode_attn with n_cached + 1 does).  0 <= n_cached < cap.
 * Both decode calls count chunk arrivals in their workspace (see "Workspaces" above): calls on different
 * workspaces are independent, whether or not they share a plan.
 */
PUREKV_API int purekv_decode_step(const purekv_plan_t* plan, const void* q_new, const void* k_new, const void* v_new,
                                  void* kc, void* vc, int32_t n_cached, int32_t cap, void* out, void* ws,
                                  size_t ws_bytes, void* stream);


/*
 * Layer stack (Sec. 3.1 and the layer-index study of the hyperparameter analysis, Sec. 4.5): which layer runs which attention and whose
 * importance estimate drives whose selection.
 *   layers 0 .. st_layer-1 run dense causal attention (Eq. 1), layers st_layer .. n_layers-1 ST-SpAttn (Sec. 3.2);
 *   layers 0 .. clie_layer also emit their recent-window column sums C (Eq. 2): a layer below clie_layer is
 *   selected with its own C (Eq. 3), layer clie_layer and every later layer with C of layer clie_layer and
 *   its own V (cross-layer importance estimation, Eq. 4).  0 <= clie_layer < st_layer <= n_layers: the estimating
 *   layer computes attention scores, so it lies below the first sparse layer.
 * purekv_stack_layer runs one layer's prefill (and importance, where the layer emits C) as the model reaches it;
 * purekv_stack_select_compact then selects and compacts all layers at once: one launch per layer below
 * clie_layer, ONE batched selection for the n_layers - clie_layer layers that share C, ONE compaction for all.
 *   q, k, v, out: that layer's tensors, as for purekv_st_spattn_prefill.   st_plan may be NULL when st_layer ==
 *   n_layers; both plans must describe the same tensor shape (dense_plan with the dense pattern).
 *   lse   fp32 [Hq, N]: scratch, needed (and overwritten) by layers <= clie_layer, else may be NULL.
 *   c_all fp32 [clie_layer + 1, Hkv, N - w]: layer l <= clie_layer writes block l.
 *   k_all, v_all: bf16, layer l at + l * kv_layer_stride elements, each [Hkv, N, d].
 *   idx_all int32 [n_layers, Hkv, h + w];  kc_all, vc_all bf16 [n_layers, Hkv, cap, d], cap >= h + w.
 *   ws: at least purekv_stack_workspace_bytes() bytes serve every call of the stack; initialise it once with
 *   purekv_stack_workspace_init (it holds the prefill workspaces of both plans, see "Workspaces" above).
 */
typedef struct {
  int32_t n_layers;   /* L >= 1                                                            */
  int32_t clie_layer; /* layer whose C is shared by itself and all later layers            */
  int32_t st_layer;   /* first ST-SpAttn layer (== n_layers: every layer dense)            */
  int32_t w, h;       /* recent window and top-h budget, as for purekv_topk_select         */
} purekv_stack_t;
PUREKV_API size_t purekv_stack_workspace_bytes(const purekv_plan_t* dense_plan, const purekv_plan_t* st_plan,
                                               const purekv_stack_t* stack);
PUREKV_API int purekv_stack_workspace_init(const purekv_plan_t* dense_plan, const purekv_plan_t* st_plan,
                                           const purekv_stack_t* stack, void* ws, size_t ws_bytes, void* stream);
PUREKV_API int purekv_stack_layer(const purekv_plan_t* dense_plan, const purekv_plan_t* st_plan,
                                  const purekv_stack_t* stack, int32_t layer, const void* q, const void* k,
                                  const void* v, void* out, float* lse, float* c_all, void* ws, size_t ws_bytes,
                                  void* stream);
PUREKV_API int purekv_stack_select_compact(const purekv_plan_t* dense_plan, const purekv_plan_t* st_plan,
                                           const purekv_stack_t* stack, const float* c_all, const void* k_all, const void* v_all,
                                           int64_t kv_layer_stride, int32_t* idx_all, void* kc_all, void* vc_all,
                                           int32_t cap, void* ws, size_t ws_bytes, void* stream);

/* Keep budget -> top-h (Sec. 3.1 keeps "the recent w tokens plus the top h"; the cache budgets of Sec. 4.2 are
 * fractions of the sequence): h = max(0, floor(ratio * n) - w), i.e. the budget counts the recent window, so that a
 * 20 % budget is exactly the paper's 5.0x compression.  The floor is taken after adding 1e-9, so that a ratio
 * like 0.29 * 100 does not lose a key to binary rounding.  Returns -1 (no valid budget) for n < 0, w < 0, or a ratio
 * that is not a finite number in [0, 1]. */
PUREKV_API int32_t purekv_budget(int32_t n, int32_t w, double ratio);

/* Work counts for reporting: flops of one prefill call counted on the (32-row block, 32-key block) pairs the
 * kernel computes (4 * 32 * 32 * d per pair and query head) and on the allowed pairs of the mask only. */
PUREKV_API double purekv_plan_kept_tile_flops(const purekv_plan_t* plan);
PUREKV_API double purekv_plan_mask_flops(const purekv_plan_t* plan);

/*
 * Board calibration (not a step of the paper's method; it exists so that the prefill kernel's rate can be read
 * against what the board sustains).  Launches, on the plan's grid of persistent workgroups (one per compute unit,
 * eight wavefronts each), a register-resident loop of the bf16 32x32x16 matrix instruction the prefill kernel uses:
 *   mix 0: the matrix instruction alone;  mix 1: each one takes an operand from a fresh 1 KB LDS fragment read;
 *   mix 2: mix 1 plus the vector work of one softmax slot (2 multiply-adds, 2 exponentials, 1 bf16 convert).
 * random_operands != 0 fills the operands with pseudo-random bf16 values, 0 with constants: the board's power
 * limit, and with it the clock, depends on how many operand bits change.  `iters` (1 .. 2^20) outer iterations of
 * 16 matrix instructions per wavefront; purekv_calib_mfma_flops gives the launch's flop count.
 *   sink  fp32 device [512 * counts[6]] (counts from purekv_plan_counts): written, values meaningless.
 *   ticks uint64 device [2]: elapsed shader cycles of wavefront 0 and the same span on the 100 MHz counter.
 * Asynchronous on `stream`, allocates nothing; the caller times it with events.  EINVAL for a host-only plan, null
 * pointers or arguments out of range.
 */
PUREKV_API int purekv_calib_mfma(const purekv_plan_t* plan, int mix, int random_operands, int32_t iters, float* sink,
                                 uint64_t* ticks, void* stream);
PUREKV_API double purekv_calib_mfma_flops(const purekv_plan_t* plan, int32_t iters);
/*
 * Second calibration loop: the skeleton of one attention tile step per compute unit (256 query rows x 64 keys,
 * head_dim 128) -- both products' MFMAs, one 1 KB LDS fragment read per fragment, the softmax vector work of every
 * score, 32 KB of K/V tile loads into LDS and one barrier per step, on pseudo-random operands; no masks, maxima,
 * tables or output.  rows_per_wavefront 32: eight wavefronts, every fragment feeds one MFMA (the prefill kernel's
 * shape); 64: four wavefronts, every fragment feeds two.  What a prefill kernel of this formulation can reach on
 * this board is read against it.
 *   src   device, 4 MiB of finite bf16 values (read as K/V tiles);  sink, ticks, iters, stream: as above.
 * purekv_calib_tile_step_flops: 4 * 256 * 64 * 128 flops per step and workgroup.
 */
PUREKV_API int purekv_calib_tile_step(const purekv_plan_t* plan, int rows_per_wavefront, int32_t iters, const void* src,
                                      float* sink, uint64_t* ticks, void* stream);
PUREKV_API double purekv_calib_tile_step_flops(const purekv_plan_t* plan, int32_t iters);

/* Static description of a status code; for PUREKV_EHIP the text of the last HIP error seen by this
 * thread is appended. */
PUREKV_API const char* purekv_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* PUREKV_H_ */

// C-ABI entry points: argument validation (host only, before any GPU call), plan life cycle, dispatch.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>

#include "common.h"

namespace purekv {

static thread_local char g_hip_msg[256] = "";

int note_hip_error(hipError_t e) {
  std::snprintf(g_hip_msg, sizeof(g_hip_msg), "HIP error %d: %s", (int)e, hipGetErrorString(e));
  return PUREKV_EHIP;
}

// Strides of one tensor (elements): {0, 0} = packed [H, N, d]; otherwise both given, rows 16-byte aligned, the token
// stride below 2^23 (the kernels multiply it with 24-bit operands) and the tensor's byte span below 2^31 (32-bit
// byte offsets).
static int resolve_strides(int64_t sh, int64_t st, int64_t heads, int64_t n, int64_t d, int64_t* out_sh, int64_t* out_st) {
  if (sh == 0 && st == 0) {
    sh = n * d;
    st = d;
  } else {
    if (st < d || (heads > 1 && sh < 1) || sh < 0) return PUREKV_EINVAL;
    if (st % 8 != 0 || sh % 8 != 0 || st >= ((int64_t)1 << 23)) return PUREKV_EINVAL;
  }
  const int64_t span = ((heads - 1) * sh + (n - 1) * st + d) * 2;
  if (span > ((int64_t)1 << 31)) return PUREKV_EINVAL;
  *out_sh = sh;
  *out_st = st;
  return PUREKV_OK;
}

static int check_shape(const purekv_shape_t* s) {
  if (s == nullptr) return PUREKV_EINVAL;
  if (s->n_frames < 1 || s->patch_h < 1 || s->patch_w < 1 || s->n_text < 0) return PUREKV_EINVAL;
  if (s->n_q_heads < 1 || s->n_kv_heads < 1 || s->n_q_heads % s->n_kv_heads != 0) return PUREKV_EINVAL;
  if (s->n_q_heads > 4096) return PUREKV_EINVAL;   // 32-bit byte offsets into the per-slice tables of split lists
  if (!(s->softmax_scale >= 0.f) || std::isinf(s->softmax_scale)) return PUREKV_EINVAL;
  const int64_t p = (int64_t)s->patch_h * s->patch_w, n = p * s->n_frames + s->n_text;
  if (p > (1 << 22) || n > (int64_t)1 << 22) return PUREKV_EINVAL;
  if (s->head_dim != 64 && s->head_dim != 128) return PUREKV_EUNSUPPORTED;
  if (s->pattern > PUREKV_PATTERN_ST) return PUREKV_EUNSUPPORTED;
  int64_t a, b;
  int rc = resolve_strides(s->q_stride_head, s->q_stride_tok, s->n_q_heads, n, s->head_dim, &a, &b);
  if (rc == PUREKV_OK) rc = resolve_strides(s->kv_stride_head, s->kv_stride_tok, s->n_kv_heads, n, s->head_dim, &a, &b);
  if (rc == PUREKV_OK) rc = resolve_strides(s->o_stride_head, s->o_stride_tok, s->n_q_heads, n, s->head_dim, &a, &b);
  return rc;
}

static int make_plan(const purekv_shape_t* s, purekv_plan_t** out, int n_cu, const uint8_t* head_mask = nullptr,
                     int32_t lse_rows = 0) {
  if (out == nullptr) return PUREKV_EINVAL;
  const int rc = check_shape(s);
  if (rc != PUREKV_OK) return rc;
  if (lse_rows < 0 || lse_rows > (int64_t)s->patch_h * s->patch_w * s->n_frames + s->n_text) return PUREKV_EINVAL;
  if (head_mask != nullptr) {   // at least one head
    bool any = false;
    for (int32_t hq = 0; hq < s->n_q_heads; ++hq) any |= head_mask[hq] != 0;
    if (!any) return PUREKV_EINVAL;
  }
  purekv_plan* p = new (std::nothrow) purekv_plan();
  if (p == nullptr) return PUREKV_ENOMEM;
  try {
    if (head_mask != nullptr) p->head_sel.assign(head_mask, head_mask + s->n_q_heads);
  } catch (const std::bad_alloc&) {
    delete p;
    return PUREKV_ENOMEM;
  }
  p->lse_rows = lse_rows;
  Geometry& g = p->g;
  g.F = s->n_frames;
  g.P = s->patch_h * s->patch_w;
  g.T = s->n_text;
  g.Nv = g.F * g.P;
  g.N = g.Nv + g.T;
  g.Hq = s->n_q_heads;
  g.Hkv = s->n_kv_heads;
  g.G = g.Hq / g.Hkv;
  g.d = s->head_dim;
  g.pattern = s->pattern;
  g.scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / std::sqrt((float)s->head_dim);
  (void)resolve_strides(s->q_stride_head, s->q_stride_tok, g.Hq, g.N, g.d, &g.q_sh, &g.q_st);
  (void)resolve_strides(s->kv_stride_head, s->kv_stride_tok, g.Hkv, g.N, g.d, &g.kv_sh, &g.kv_st);
  (void)resolve_strides(s->o_stride_head, s->o_stride_tok, g.Hq, g.N, g.d, &g.o_sh, &g.o_st);
  try {
    build_plan(*p, n_cu);
  } catch (const std::bad_alloc&) {
    delete p;
    return PUREKV_ENOMEM;
  }
  *out = p;
  return PUREKV_OK;
}

static bool launchable(const purekv_plan_t* p) { return p != nullptr && p->d_stream != nullptr; }

}  // namespace purekv

using namespace purekv;

extern "C" {

int purekv_plan_create_host(const purekv_shape_t* shape, int32_t n_workgroups, purekv_plan_t** out) {
  if (n_workgroups < 1 || n_workgroups > 65536) return PUREKV_EINVAL;
  return make_plan(shape, out, n_workgroups);
}

static int create_on_device(const purekv_shape_t* shape, const uint8_t* head_mask, int32_t lse_rows, purekv_plan_t** out,
                            void* stream);

int purekv_plan_create(const purekv_shape_t* shape, purekv_plan_t** out, void* stream) {
  return create_on_device(shape, nullptr, 0, out, stream);
}

int purekv_plan_create_window(const purekv_shape_t* shape, int32_t w, purekv_plan_t** out, void* stream) {
  if (w < 1) return PUREKV_EINVAL;
  return create_on_device(shape, nullptr, w, out, stream);
}

int purekv_plan_create_window_host(const purekv_shape_t* shape, int32_t w, int32_t n_workgroups, purekv_plan_t** out) {
  if (w < 1 || n_workgroups < 1 || n_workgroups > 65536) return PUREKV_EINVAL;
  return make_plan(shape, out, n_workgroups, nullptr, w);
}

int purekv_plan_create_heads(const purekv_shape_t* shape, const uint8_t* head_mask, purekv_plan_t** out, void* stream) {
  if (head_mask == nullptr) return PUREKV_EINVAL;
  return create_on_device(shape, head_mask, 0, out, stream);
}

int purekv_plan_create_heads_host(const purekv_shape_t* shape, const uint8_t* head_mask, int32_t n_workgroups,
                                  purekv_plan_t** out) {
  if (head_mask == nullptr || n_workgroups < 1 || n_workgroups > 65536) return PUREKV_EINVAL;
  return make_plan(shape, out, n_workgroups, head_mask);
}

static int create_on_device(const purekv_shape_t* shape, const uint8_t* head_mask, int32_t lse_rows, purekv_plan_t** out,
                            void* stream) {
  if (out == nullptr) return PUREKV_EINVAL;
  int rc = check_shape(shape);
  if (rc != PUREKV_OK) return rc;
  int dev = 0, n_cu = 256;
  PUREKV_HIP_TRY(hipGetDevice(&dev));
  PUREKV_HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev));
  purekv_plan_t* p = nullptr;
  rc = make_plan(shape, &p, n_cu > 0 ? n_cu : 256, head_mask, lse_rows);
  if (rc != PUREKV_OK) return rc;
  p->device = dev;
  rc = static_score_buffer(dev, &p->d_static_scores);
  if (rc != PUREKV_OK) {
    delete p;
    return rc;
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t sb = p->stream.size() * sizeof(StreamEntry), ub = p->units.size() * sizeof(Unit),
               qb = p->queue_begin.size() * sizeof(int32_t);
  hipError_t e = hipMalloc(reinterpret_cast<void**>(&p->d_stream), sb ? sb : 16);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->d_units), ub ? ub : 16);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->d_queue_begin), qb ? qb : 16);
  if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void**>(&p->d_queue_unit0), qb ? qb : 16);
  if (e == hipSuccess && sb) e = hipMemcpyAsync(p->d_stream, p->stream.data(), sb, hipMemcpyHostToDevice, st);
  if (e == hipSuccess && ub) e = hipMemcpyAsync(p->d_units, p->units.data(), ub, hipMemcpyHostToDevice, st);
  if (e == hipSuccess && qb) e = hipMemcpyAsync(p->d_queue_begin, p->queue_begin.data(), qb, hipMemcpyHostToDevice, st);
  if (e == hipSuccess && qb)
    e = hipMemcpyAsync(p->d_queue_unit0, p->queue_units_begin.data(), qb, hipMemcpyHostToDevice, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);  // the host vectors must outlive the copies: finish them now
  if (e != hipSuccess) {
    purekv_plan_destroy(p);
    return note_hip_error(e);
  }
  *out = p;
  return PUREKV_OK;
}

int purekv_plan_destroy(purekv_plan_t* p) {
  if (p == nullptr) return PUREKV_OK;
  if (p->d_stream) (void)hipFree(p->d_stream);
  if (p->d_units) (void)hipFree(p->d_units);
  if (p->d_queue_begin) (void)hipFree(p->d_queue_begin);
  if (p->d_queue_unit0) (void)hipFree(p->d_queue_unit0);
  delete p;
  return PUREKV_OK;
}

int purekv_plan_counts(const purekv_plan_t* p, int64_t counts[16]) {
  if (p == nullptr || counts == nullptr) return PUREKV_EINVAL;
  counts[0] = p->g.N;
  counts[1] = p->n_qtiles;
  counts[2] = (int64_t)p->items.size();
  counts[3] = (int64_t)p->tiles.size();
  counts[4] = p->n_blocks;
  counts[5] = (int64_t)p->merges.size();
  counts[6] = p->n_queues;
  counts[7] = p->g.R;
  counts[8] = p->g.Gs;
  counts[9] = p->g.n_groups;
  for (int k = 0; k < 4; ++k) counts[10 + k] = p->n_kind[k];
  counts[14] = p->lse_rows;
  counts[15] = p->lse_queue0;
  return PUREKV_OK;
}

int purekv_plan_qtile_list(const purekv_plan_t* p, int32_t qt, int32_t* refs, int32_t cap) {
  if (p == nullptr || qt < 0 || qt >= p->n_qtiles || cap < 0 || (cap > 0 && refs == nullptr)) return PUREKV_EINVAL;
  const int32_t b = p->qtile_begin[qt], len = p->qtile_begin[qt + 1] - b;
  for (int32_t i = 0; i < len && i < cap; ++i) {
    refs[3 * i] = p->tiles[b + i].tile;
    refs[3 * i + 1] = (int32_t)p->tiles[b + i].need;
    refs[3 * i + 2] = (int32_t)p->tiles[b + i].kinds;
  }
  return len;
}

int purekv_plan_queue(const purekv_plan_t* p, int32_t wg, int32_t* units, int32_t cap) {
  if (p == nullptr || wg < 0 || wg >= p->n_queues || cap < 0 || (cap > 0 && units == nullptr)) return PUREKV_EINVAL;
  const int32_t b = p->queue_units_begin[wg], len = p->queue_units_begin[wg + 1] - b;
  for (int32_t i = 0; i < len && i < cap; ++i) {
    units[2 * i] = p->queue_units[2 * (b + i)];
    units[2 * i + 1] = p->queue_units[2 * (b + i) + 1];
  }
  return len;
}

int purekv_plan_steps(const purekv_plan_t* p, int32_t wg, int32_t* steps, int32_t cap) {
  if (p == nullptr || wg < 0 || wg >= p->n_queues || cap < 0 || (cap > 0 && steps == nullptr)) return PUREKV_EINVAL;
  const int32_t b = p->queue_begin[wg], len = p->queue_begin[wg + 1] - b;
  for (int32_t i = 0; i < len && i < cap; ++i) {
    const StreamEntry& e = p->stream[b + i];
    const int32_t rec[4] = {(int32_t)e.kv_off, (int32_t)e.need, (int32_t)e.kinds, e.k0};
    for (int k = 0; k < 4; ++k) steps[4 * i + k] = rec[k];
  }
  return len;
}

int purekv_plan_item(const purekv_plan_t* p, int32_t it, int32_t item[6]) {
  if (p == nullptr || item == nullptr || it < 0 || it >= (int32_t)p->items.size()) return PUREKV_EINVAL;
  const WorkItem& w = p->items[it];
  item[0] = w.qtile;
  item[1] = w.list_begin;
  item[2] = w.n_tiles;
  item[3] = w.split;
  item[4] = w.n_splits;
  item[5] = w.slot;
  return PUREKV_OK;
}

double purekv_plan_kept_tile_flops(const purekv_plan_t* p) {
  if (p == nullptr) return 0.0;
  return 4.0 * kBlockRows * kBlockKeys * p->g.d * (double)p->n_blocks * p->n_heads_sel;
}

double purekv_plan_mask_flops(const purekv_plan_t* p) {
  if (p == nullptr) return 0.0;
  return 4.0 * p->g.d * p->mask_pairs * p->n_heads_sel;
}

size_t purekv_workspace_bytes(const purekv_plan_t* p, int op, int32_t n_layers, int32_t w, int32_t cap) {
  if (p == nullptr) return 0;
  switch (op) {
    case PUREKV_OP_PREFILL:
      return prefill_ws_bytes(*p);
    case PUREKV_OP_TOPK:
      return (n_layers >= 1 && w >= 1 && w <= p->g.N) ? topk_ws_bytes(*p, n_layers, w) : 0;
    case PUREKV_OP_DECODE:
      return cap >= 1 ? decode_ws_bytes(*p, cap) : 0;
    default:
      return 0;
  }
}

int purekv_workspace_init(const purekv_plan_t* p, int op, void* ws, size_t ws_bytes, int32_t n_layers, int32_t w,
                          int32_t cap, void* stream) {
  if (!launchable(p)) return PUREKV_EINVAL;
  if (op < PUREKV_OP_PREFILL || op > PUREKV_OP_DECODE) return PUREKV_EINVAL;
  const size_t need = purekv_workspace_bytes(p, op, n_layers, w, cap);
  if (need == 0) return PUREKV_OK;
  if (ws == nullptr || ws_bytes < need) return PUREKV_EWORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (op == PUREKV_OP_PREFILL) return launch_prefill_ws_init(*p, ws, st);
  if (op == PUREKV_OP_DECODE) return launch_decode_ws_init(*p, ws, st);
  return PUREKV_OK;   // the other workspaces hold nothing that outlives a call
}

int purekv_st_spattn_prefill(const purekv_plan_t* p, const void* q, const void* k, const void* v, void* out,
                             float* lse, void* ws, size_t ws_bytes, void* stream) {
  if (!launchable(p) || q == nullptr || k == nullptr || v == nullptr || out == nullptr) return PUREKV_EINVAL;
  const size_t need = prefill_ws_bytes(*p);
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return PUREKV_EWORKSPACE;
  return launch_prefill(*p, q, k, v, out, lse, nullptr, ws, static_cast<hipStream_t>(stream));
}

int purekv_st_spattn_prefill_vnorm(const purekv_plan_t* p, const void* q, const void* k, const void* v, void* out,
                                   float* lse, float* vnorm2, void* ws, size_t ws_bytes, void* stream) {
  if (!launchable(p) || q == nullptr || k == nullptr || v == nullptr || out == nullptr || vnorm2 == nullptr)
    return PUREKV_EINVAL;
  const size_t need = prefill_ws_bytes(*p);
  if (need > 0 && (ws == nullptr || ws_bytes < need)) return PUREKV_EWORKSPACE;
  return launch_prefill(*p, q, k, v, out, lse, vnorm2, ws, static_cast<hipStream_t>(stream));
}

int purekv_topk_select_vnorm(const purekv_plan_t* p, const float* c, const float* vnorm2, int64_t vn_layer_stride,
                             int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws,
                             size_t ws_bytes, void* stream) {
  if (!launchable(p) || idx_out == nullptr || vnorm2 == nullptr || n_layers < 1) return PUREKV_EINVAL;
  if (w < 1 || w > p->g.N || h < 0 || h > p->g.N - w) return PUREKV_EINVAL;
  if (c == nullptr && w < p->g.N) return PUREKV_EINVAL;
  if (n_layers > 1 && vn_layer_stride < (int64_t)p->g.Hkv * p->g.N) return PUREKV_EINVAL;
  if (s_out == nullptr) {
    const size_t need = topk_ws_bytes(*p, n_layers, w);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return PUREKV_EWORKSPACE;
  }
  return launch_topk_norms(*p, c, vnorm2, vn_layer_stride, n_layers, w, h, idx_out, s_out, ws,
                           static_cast<hipStream_t>(stream));
}

int purekv_lowlayer_importance(const purekv_plan_t* p, const void* q, const void* k, const float* lse, int32_t w,
                               float* c_out, void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  if (!launchable(p) || q == nullptr || k == nullptr || lse == nullptr) return PUREKV_EINVAL;
  if (w < 1 || w > p->g.N) return PUREKV_EINVAL;
  if (p->lse_rows > 0 && w > p->lse_rows) return PUREKV_EINVAL;   // a window plan's prefill wrote fewer rows of lse
  if (c_out == nullptr && w < p->g.N) return PUREKV_EINVAL;
  return launch_importance(*p, q, k, lse, w, c_out, static_cast<hipStream_t>(stream));
}

int purekv_spearman(const float* s_hat, const float* s, int32_t n_rows, int32_t n_keys, uint64_t* sum_d2_out,
                    double* rho_out, void* stream) {
  if (s_hat == nullptr || s == nullptr || sum_d2_out == nullptr) return PUREKV_EINVAL;
  if (n_rows < 1 || n_rows > 65535 || n_keys < 2 || n_keys > 131072) return PUREKV_EINVAL;
  return launch_spearman(s_hat, s, n_rows, n_keys, sum_d2_out, rho_out, static_cast<hipStream_t>(stream));
}

int purekv_topk_select(const purekv_plan_t* p, const float* c, const void* v, int64_t v_layer_stride,
                       int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, float* s_out, void* ws,
                       size_t ws_bytes, void* stream) {
  if (!launchable(p) || idx_out == nullptr || n_layers < 1) return PUREKV_EINVAL;
  if (w < 1 || w > p->g.N || h < 0 || h > p->g.N - w) return PUREKV_EINVAL;
  if (c == nullptr && w < p->g.N) return PUREKV_EINVAL;
  if (v == nullptr && n_layers != 1) return PUREKV_EINVAL;
  if (v != nullptr && n_layers > 1 && v_layer_stride < 1) return PUREKV_EINVAL;
  if (v != nullptr && s_out == nullptr) {
    const size_t need = topk_ws_bytes(*p, n_layers, w);
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return PUREKV_EWORKSPACE;
  }
  return launch_topk(*p, c, v, v_layer_stride, n_layers, w, h, idx_out, s_out, ws, static_cast<hipStream_t>(stream));
}

int purekv_topk_select_static(const purekv_plan_t* p, const float* c, const void* v, int64_t v_layer_stride,
                              int32_t n_layers, int32_t w, int32_t h, int32_t* idx_out, void* stream) {
  if (!launchable(p) || idx_out == nullptr || n_layers < 1) return PUREKV_EINVAL;
  if (w < 1 || w > p->g.N || h < 0 || h > p->g.N - w) return PUREKV_EINVAL;
  if (c == nullptr && w < p->g.N) return PUREKV_EINVAL;
  if (v == nullptr && n_layers != 1) return PUREKV_EINVAL;
  if (v != nullptr && n_layers > 1 && v_layer_stride < 1) return PUREKV_EINVAL;
  if (v != nullptr && (size_t)n_layers * p->g.Hkv * (size_t)(p->g.N - w) > topk_static_capacity_floats())
    return PUREKV_EWORKSPACE;   // the scores do not fit the static buffer: use purekv_topk_select with a workspace
  if (p->d_static_scores == nullptr) return PUREKV_EINVAL;
  return launch_topk(*p, c, v, v_layer_stride, n_layers, w, h, idx_out, nullptr, p->d_static_scores,
                     static_cast<hipStream_t>(stream));
}

int purekv_kv_compact(const purekv_plan_t* p, const void* k, const void* v, int64_t kv_layer_stride, int32_t n_layers,
                      const int32_t* idx, int32_t n_keep, void* kc, void* vc, int32_t cap, void* stream) {
  if (!launchable(p) || k == nullptr || v == nullptr || kc == nullptr || vc == nullptr || n_layers < 1)
    return PUREKV_EINVAL;
  if (n_keep < 0 || n_keep > cap || cap < 1 || n_keep > p->g.N) return PUREKV_EINVAL;
  if (idx == nullptr && n_keep > 0) return PUREKV_EINVAL;
  if (n_layers > 1 && kv_layer_stride < 1) return PUREKV_EINVAL;
  return launch_compact(*p, k, v, kv_layer_stride, n_layers, idx, n_keep, kc, vc, cap, static_cast<hipStream_t>(stream));
}

int purekv_kv_append(const purekv_plan_t* p, const void* k_new, const void* v_new, void* kc, void* vc,
                     int32_t n_cached, int32_t cap, void* stream) {
  if (!launchable(p) || k_new == nullptr || v_new == nullptr || kc == nullptr || vc == nullptr) return PUREKV_EINVAL;
  if (n_cached < 0 || n_cached >= cap) return PUREKV_EINVAL;
  return launch_append(*p, k_new, v_new, kc, vc, n_cached, cap, static_cast<hipStream_t>(stream));
}

int purekv_decode_attn(const purekv_plan_t* p, const void* q_new, const void* kc, const void* vc, int32_t n_cached,
                       int32_t cap, void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!launchable(p) || q_new == nullptr || kc == nullptr || vc == nullptr || out == nullptr) return PUREKV_EINVAL;
  if (n_cached < 1 || n_cached > cap) return PUREKV_EINVAL;
  if (ws == nullptr || ws_bytes < decode_ws_bytes(*p, cap)) return PUREKV_EWORKSPACE;
  return launch_decode(*p, q_new, nullptr, nullptr, const_cast<void*>(kc), const_cast<void*>(vc), n_cached, cap, out, ws,
                       static_cast<hipStream_t>(stream));
}

int purekv_decode_step(const purekv_plan_t* p, const void* q_new, const void* k_new, const void* v_new, void* kc,
                       void* vc, int32_t n_cached, int32_t cap, void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!launchable(p) || q_new == nullptr || k_new == nullptr || v_new == nullptr || kc == nullptr || vc == nullptr ||
      out == nullptr)
    return PUREKV_EINVAL;
  if (n_cached < 0 || n_cached >= cap) return PUREKV_EINVAL;
  if (ws == nullptr || ws_bytes < decode_ws_bytes(*p, cap)) return PUREKV_EWORKSPACE;
  return launch_decode(*p, q_new, k_new, v_new, kc, vc, n_cached + 1, cap, out, ws, static_cast<hipStream_t>(stream));
}

// ---- layer stack: which layer runs which attention, which C drives which layer's selection ----
static int check_stack(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s) {
  if (!launchable(dense) || s == nullptr) return PUREKV_EINVAL;
  if (s->n_layers < 1 || s->clie_layer < 0 || s->clie_layer >= s->st_layer || s->st_layer > s->n_layers)
    return PUREKV_EINVAL;
  const Geometry& a = dense->g;
  if (a.pattern != PUREKV_PATTERN_DENSE) return PUREKV_EINVAL;
  if (s->w < 1 || s->w > a.N || s->h < 0 || s->h > a.N - s->w) return PUREKV_EINVAL;
  if (s->st_layer < s->n_layers) {   // a sparse plan is needed and must describe the same tensors
    if (!launchable(st)) return PUREKV_EINVAL;
    const Geometry& b = st->g;
    if (a.N != b.N || a.Nv != b.Nv || a.P != b.P || a.Hq != b.Hq || a.Hkv != b.Hkv || a.d != b.d || a.scale != b.scale ||
        a.q_sh != b.q_sh || a.q_st != b.q_st || a.kv_sh != b.kv_sh || a.kv_st != b.kv_st || a.o_sh != b.o_sh ||
        a.o_st != b.o_st || dense->device != st->device)
      return PUREKV_EINVAL;
  }
  return PUREKV_OK;
}

// One buffer serves every call of a stack: [prefill workspace of the dense plan][prefill workspace of the sparse
// plan][scores of the selection].  The three parts are disjoint because the prefill workspaces begin with arrival
// counters that must stay zero between calls: nothing else may ever write there.
struct StackWs {
  size_t st_off = 0, scores_off = 0, total = 0;
};
static StackWs stack_ws_layout(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s) {
  auto up = [](size_t x) { return (x + 255) / 256 * 256; };
  StackWs l;
  l.st_off = up(prefill_ws_bytes(*dense));
  l.scores_off = l.st_off + (s->st_layer < s->n_layers ? up(prefill_ws_bytes(*st)) : 0);
  l.total = l.scores_off + topk_ws_bytes(*dense, s->n_layers - s->clie_layer, s->w);
  return l;
}

size_t purekv_stack_workspace_bytes(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s) {
  if (check_stack(dense, st, s) != PUREKV_OK) return 0;
  return stack_ws_layout(dense, st, s).total;
}

int purekv_stack_workspace_init(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s, void* ws,
                                size_t ws_bytes, void* stream) {
  const int rc = check_stack(dense, st, s);
  if (rc != PUREKV_OK) return rc;
  const StackWs l = stack_ws_layout(dense, st, s);
  if (l.total == 0) return PUREKV_OK;
  if (ws == nullptr || ws_bytes < l.total) return PUREKV_EWORKSPACE;
  hipStream_t sm = static_cast<hipStream_t>(stream);
  int r = launch_prefill_ws_init(*dense, ws, sm);
  if (r == PUREKV_OK && s->st_layer < s->n_layers) r = launch_prefill_ws_init(*st, static_cast<char*>(ws) + l.st_off, sm);
  return r;
}

int purekv_stack_layer(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s, int32_t layer,
                       const void* q, const void* k, const void* v, void* out, float* lse, float* c_all, void* ws,
                       size_t ws_bytes, void* stream) {
  const int rc = check_stack(dense, st, s);
  if (rc != PUREKV_OK) return rc;
  if (layer < 0 || layer >= s->n_layers || q == nullptr || k == nullptr || v == nullptr || out == nullptr)
    return PUREKV_EINVAL;
  const bool sparse = layer >= s->st_layer, emits_c = layer <= s->clie_layer;
  const purekv_plan_t* p = sparse ? st : dense;
  const int n_keys = p->g.N - s->w;
  if (emits_c && (lse == nullptr || (c_all == nullptr && n_keys > 0))) return PUREKV_EINVAL;
  const StackWs lay = stack_ws_layout(dense, st, s);
  if (lay.total > 0 && (ws == nullptr || ws_bytes < lay.total)) return PUREKV_EWORKSPACE;
  if (ws != nullptr && sparse) ws = static_cast<char*>(ws) + lay.st_off;
  hipStream_t sm = static_cast<hipStream_t>(stream);
  const int rp = launch_prefill(*p, q, k, v, out, emits_c ? lse : nullptr, nullptr, ws, sm);
  if (rp != PUREKV_OK || !emits_c) return rp;
  return launch_importance(*p, q, k, lse, s->w, c_all + (size_t)layer * p->g.Hkv * n_keys, sm);
}

int purekv_stack_select_compact(const purekv_plan_t* dense, const purekv_plan_t* st, const purekv_stack_t* s,
                                const float* c_all, const void* k_all, const void* v_all, int64_t kv_layer_stride,
                                int32_t* idx_all, void* kc_all, void* vc_all, int32_t cap, void* ws, size_t ws_bytes,
                                void* stream) {
  const int rcs = check_stack(dense, st, s);
  if (rcs != PUREKV_OK) return rcs;
  const Geometry& g = dense->g;
  const int n_keys = g.N - s->w, n_keep = s->h + s->w, L = s->n_layers, n_shared = L - s->clie_layer;
  if (k_all == nullptr || v_all == nullptr || idx_all == nullptr || kc_all == nullptr || vc_all == nullptr)
    return PUREKV_EINVAL;
  if (c_all == nullptr && n_keys > 0) return PUREKV_EINVAL;
  if (cap < n_keep) return PUREKV_EINVAL;
  if (L > 1 && kv_layer_stride < 1) return PUREKV_EINVAL;
  // the same buffer the layers used: the scores go behind the prefill counters (see stack_ws_layout)
  const size_t scores_off = stack_ws_layout(dense, st, s).scores_off;
  const size_t need = topk_ws_bytes(*dense, n_shared, s->w);
  if (need > 0 && (ws == nullptr || ws_bytes < scores_off + need)) return PUREKV_EWORKSPACE;
  ws = static_cast<char*>(ws) + scores_off;
  hipStream_t sm = static_cast<hipStream_t>(stream);
  const uint16_t* vb = static_cast<const uint16_t*>(v_all);
  const size_t c_stride = (size_t)g.Hkv * n_keys, idx_stride = (size_t)g.Hkv * n_keep;
  // layers below the estimating one have attention scores of their own (Eq. 3) ...
  for (int l = 0; l < s->clie_layer; ++l) {
    const int rc = launch_topk(*dense, c_all + l * c_stride, vb + (size_t)l * kv_layer_stride, 0, 1, s->w, s->h,
                               idx_all + l * idx_stride, nullptr, ws, sm);
    if (rc != PUREKV_OK) return rc;
  }
  // ... it and every later layer share its C, each with its own V (Eq. 4): one batched call
  const int rc = launch_topk(*dense, c_all + (size_t)s->clie_layer * c_stride, vb + (size_t)s->clie_layer * kv_layer_stride,
                             kv_layer_stride, n_shared, s->w, s->h, idx_all + (size_t)s->clie_layer * idx_stride, nullptr,
                             ws, sm);
  if (rc != PUREKV_OK) return rc;
  return launch_compact(*dense, k_all, v_all, kv_layer_stride, L, idx_all, n_keep, kc_all, vc_all, cap, sm);
}

int purekv_calib_mfma(const purekv_plan_t* p, int mix, int random_operands, int32_t iters, float* sink, uint64_t* ticks,
                      void* stream) {
  if (!launchable(p) || sink == nullptr || ticks == nullptr) return PUREKV_EINVAL;
  if (mix < 0 || mix > 2 || iters < 1 || iters > (1 << 20)) return PUREKV_EINVAL;
  return launch_calib_mfma(*p, mix, random_operands != 0, iters, sink, ticks, static_cast<hipStream_t>(stream));
}

int purekv_calib_tile_step(const purekv_plan_t* p, int rows_per_wavefront, int32_t iters, const void* src, float* sink,
                           uint64_t* ticks, void* stream) {
  if (!launchable(p) || src == nullptr || sink == nullptr || ticks == nullptr) return PUREKV_EINVAL;
  if ((rows_per_wavefront != 32 && rows_per_wavefront != 64) || iters < 1 || iters > (1 << 20)) return PUREKV_EINVAL;
  return launch_calib_step(*p, rows_per_wavefront, iters, src, sink, ticks, static_cast<hipStream_t>(stream));
}

double purekv_calib_tile_step_flops(const purekv_plan_t* p, int32_t iters) {
  return (p == nullptr || iters < 1) ? 0.0 : calib_step_flops(*p, iters);
}

double purekv_calib_mfma_flops(const purekv_plan_t* p, int32_t iters) {
  return (p == nullptr || iters < 1) ? 0.0 : calib_mfma_flops(*p, iters);
}

int32_t purekv_budget(int32_t n, int32_t w, double ratio) {
  if (n < 0 || w < 0 || !std::isfinite(ratio) || ratio < 0.0 || ratio > 1.0) return -1;
  const double kept = std::floor(ratio * (double)n + 1e-9);   // 0.29 * 100 is 28.999999999999996 in binary
  const int64_t h = (int64_t)kept - w;
  return h > 0 ? (int32_t)h : 0;
}

const char* purekv_strerror(int status) {
  static thread_local char buf[320];
  switch (status) {
    case PUREKV_OK:
      return "ok";
    case PUREKV_EINVAL:
      return "invalid argument (null pointer, size out of range, inconsistent shape, or a host-only plan)";
    case PUREKV_EUNSUPPORTED:
      return "unsupported shape (head_dim must be 64 or 128; pattern must be 0..3)";
    case PUREKV_EWORKSPACE:
      return "workspace missing or smaller than purekv_workspace_bytes()";
    case PUREKV_ENOMEM:
      return "host allocation failed";
    case PUREKV_EHIP:
      std::snprintf(buf, sizeof(buf), "HIP runtime failure: %s", g_hip_msg[0] ? g_hip_msg : "(no detail recorded)");
      return buf;
    default:
      return "unknown status";
  }
}

}  // extern "C"

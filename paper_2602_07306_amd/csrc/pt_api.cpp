// Host side of libpt: configuration checks, arena layout, and the launch sequence of
// Algorithm 1 (Section 2.2 of the paper) for prefill and KV-cached decode.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "pt_internal.h"

static thread_local char g_err[512] = "";
static bool g_fold_rmsnorm = true;   // pt_set_tuning(PT_TUNE_FOLD_RMSNORM)

int pt_set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

extern "C" const char* pt_last_error(void) { return g_err; }

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int pt_validate_config(const pt_config* c) {
  if (!c) return pt_set_error(PT_ERR_NULL_POINTER, "config is NULL");
  if (c->n_tracks < 1 || c->n_tracks > 16)
    return pt_set_error(PT_ERR_INVALID_CONFIG, "n_tracks = %d, need 1..16", c->n_tracks);
  if (c->n_layers < 1 || c->block_depth < 1)
    return pt_set_error(PT_ERR_INVALID_CONFIG, "n_layers and block_depth must be >= 1");
  if (c->n_layers % c->block_depth != 0)
    return pt_set_error(PT_ERR_INVALID_CONFIG,
                        "n_layers (%d) is not a multiple of block_depth (%d): the output of "
                        "Algorithm 1 is only defined by a merge", c->n_layers, c->block_depth);
  if (c->d_model < 8 || c->d_model % 8) return pt_set_error(PT_ERR_INVALID_CONFIG, "d_model must be a positive multiple of 8");
  if (c->head_dim < 8 || c->head_dim % 8 || c->head_dim > 256)
    return pt_set_error(PT_ERR_INVALID_CONFIG, "head_dim must be a multiple of 8 in 8..256");
  if (c->n_heads < 1 || c->n_kv_heads < 1 || c->n_heads % c->n_kv_heads)
    return pt_set_error(PT_ERR_INVALID_CONFIG, "n_kv_heads (%d) must divide n_heads (%d)", c->n_kv_heads, c->n_heads);
  if (c->d_ffn < 32 || c->d_ffn % 32) return pt_set_error(PT_ERR_INVALID_CONFIG, "d_ffn must be a positive multiple of 32");
  if (c->vocab < 0 || c->vocab % 8) return pt_set_error(PT_ERR_INVALID_CONFIG, "vocab must be 0 or a positive multiple of 8");
  if (c->max_batch < 1 || c->max_seq < 1) return pt_set_error(PT_ERR_INVALID_CONFIG, "max_batch and max_seq must be >= 1");
  if ((int64_t)c->max_batch * c->max_seq > (int64_t)1 << 30)
    return pt_set_error(PT_ERR_INVALID_CONFIG, "max_batch * max_seq too large");
  if (c->dtype != PT_F32 && c->dtype != PT_BF16) return pt_set_error(PT_ERR_INVALID_CONFIG, "dtype must be PT_F32 or PT_BF16");
  if (c->n_experts < 0 || c->n_experts > 64) return pt_set_error(PT_ERR_INVALID_CONFIG, "n_experts = %d, need 0 (dense) or 1..64", c->n_experts);
  if (c->n_experts == 0 && c->top_k != 0) return pt_set_error(PT_ERR_INVALID_CONFIG, "top_k must be 0 for a dense model");
  if (c->n_experts > 0 && (c->top_k < 1 || c->top_k > 8 || c->top_k > c->n_experts))
    return pt_set_error(PT_ERR_INVALID_CONFIG, "top_k = %d, need 1..min(8, n_experts)", c->top_k);
  if (c->n_experts > 0 && c->n_layers >= 4096) return pt_set_error(PT_ERR_INVALID_CONFIG, "a PT-MoE model needs n_layers < 4096");
  if (!(c->rms_eps >= 0.f) || !(c->rope_theta > 0.f) || !(c->init_std >= 0.f) || !(c->merge_scale == c->merge_scale))
    return pt_set_error(PT_ERR_INVALID_CONFIG, "rms_eps, rope_theta, init_std or merge_scale out of range");
  return PT_OK;
}

int pt_compute_layout(const pt_config* c, pt_layout* l) {
  memset(l, 0, sizeof(*l));
  const int64_t T = c->n_tracks, L = c->n_layers, d = c->d_model, f = c->d_ffn, hd = c->head_dim;
  const int64_t es = c->dtype == PT_F32 ? 4 : 2;
  l->elem_size = (int32_t)es;
  l->hq = (int64_t)c->n_heads * hd;
  l->hk = (int64_t)c->n_kv_heads * hd;
  l->n_qkv = l->hq + 2 * l->hk;
  auto up = [](int64_t x) { return (x + 127) / 128 * 128; };
  l->wqkv_elems = up(l->n_qkv * d);
  l->wo_elems = up(d * l->hq);
  l->wgu_elems = up(2 * f * d);
  l->wd_elems = up(d * f);
  l->e_pad = (c->n_experts + 3) / 4 * 4;
  l->wr_elems = up(l->e_pad * d);
  l->expert_elems = l->wgu_elems + l->wd_elems;
  l->off_wr_elems = l->wqkv_elems + l->wo_elems;
  l->off_exp_elems = l->off_wr_elems + l->wr_elems;
  l->layer_w_elems = l->off_exp_elems + (c->n_experts > 0 ? c->n_experts : 1) * l->expert_elems;
  size_t off = 0;
  l->off_layers = off; off = align_up(off + (size_t)(T * L * l->layer_w_elems * es), 256);
  l->off_gains = off;  off = align_up(off + (size_t)(T * L * 2 * d * 4), 256);
  l->off_gf = off;     off = align_up(off + (size_t)(d * 4), 256);
  l->off_embed = off;  off = align_up(off + (size_t)((int64_t)c->vocab * d * es), 256);
  l->off_headT = off;  off = align_up(off + (size_t)((int64_t)c->vocab * d * es), 256);
  l->s_k = (c->max_seq + 63) / 64 * 64;
  l->off_rope = off;   off = align_up(off + (size_t)(l->s_k * hd * 4), 256);
  l->off_flag = off;   off = align_up(off + 4, 256);
  l->weight_bytes = off;

  l->s_pad = l->s_k + 64;
  const int64_t B = c->max_batch;
  const int64_t k_head = l->s_k * hd, v_head = hd * l->s_pad;
  l->off_k = 0;
  l->off_v = align_up((size_t)(T * L * B * c->n_kv_heads * k_head * es), 256);
  l->off_seq = align_up(l->off_v + (size_t)(T * L * B * c->n_kv_heads * v_head * es), 256);
  l->kv_bytes = align_up(l->off_seq + (size_t)(B * 16), 256);

  pt_workspace w;
  pt_layout_workspace(c, l, B * l->s_k, B, PT_SK_PART_FLOATS, PT_MAX_SPLITS, &w);
  l->ws_bytes = w.bytes;
  (void)f;
  return PT_OK;
}

void pt_layout_workspace(const pt_config* c, const pt_layout* l, int64_t rows, int64_t batch, int64_t skp_floats,
                         int32_t max_splits, pt_workspace* w) {
  const int64_t T = c->n_tracks, d = c->d_model, f = c->d_ffn, hd = c->head_dim, es = l->elem_size;
  size_t off = 0;
  w->base = nullptr;
  w->off_h = off;    off = align_up(off + (size_t)(T * rows * d * 4), 256);
  w->off_hm = off;   off = align_up(off + (size_t)(rows * d * 4), 256);
  w->off_a = off;    off = align_up(off + (size_t)(T * rows * d * es), 256);
  w->off_q = off;    off = align_up(off + (size_t)(T * rows * l->hq * es), 256);
  w->off_o = off;    off = align_up(off + (size_t)(T * rows * l->hq * es), 256);
  const int64_t E = c->n_experts, k = c->top_k;
  w->slots = E > 0 ? (rows * k + E * 255 + 255) / 256 * 256 : 0;
  w->off_m = off;    off = align_up(off + (size_t)(T * (E > 0 ? w->slots : rows) * f * es), 256);
  w->off_part = off; off = align_up(off + (size_t)(T * batch * c->n_heads * max_splits * (hd + 2) * 4), 256);
  w->off_ss = off;   off = align_up(off + (size_t)(T * rows * ((d + 63) / 64) * 4), 256);
  w->off_rinv = off; off = align_up(off + (size_t)(T * rows * 4), 256);
  w->off_rowmap = off; off = align_up(off + (size_t)(rows * 8), 256);
  w->off_rowidx = off; off = align_up(off + (size_t)((batch + rows) * 4), 256);
  w->off_rlogit = w->off_route = w->off_gate = w->off_slot = w->off_perm = w->off_blk = w->off_cnt = w->off_y = 0;
  if (E > 0) {
    w->off_rlogit = off; off = align_up(off + (size_t)(T * rows * l->e_pad * 4), 256);
    w->off_route = off;  off = align_up(off + (size_t)(T * rows * k * 4), 256);
    w->off_gate = off;   off = align_up(off + (size_t)(T * rows * k * 4), 256);
    w->off_slot = off;   off = align_up(off + (size_t)(T * rows * k * 4), 256);
    w->off_perm = off;   off = align_up(off + (size_t)(T * w->slots * 4), 256);
    w->off_blk = off;    off = align_up(off + (size_t)(T * (w->slots / 64) * 4), 256);
    w->off_cnt = off;    off = align_up(off + (size_t)(T * ((rows + 255) / 256 + 2) * 64 * 4), 256);
    w->off_y = off;      off = align_up(off + (size_t)(T * w->slots * d * 4), 256);
  }
  w->off_skp = off;  off = align_up(off + (size_t)skp_floats * 4, 256);
  w->bytes = off;
  w->skp_floats = skp_floats;
  w->max_splits = max_splits;
}

extern "C" int pt_query_bytes(const pt_config* cfg, size_t* w, size_t* kv, size_t* ws) {
  int rc = pt_validate_config(cfg);
  if (rc) return rc;
  pt_layout l;
  pt_compute_layout(cfg, &l);
  if (w) *w = l.weight_bytes;
  if (kv) *kv = l.kv_bytes;
  if (ws) *ws = l.ws_bytes;
  return PT_OK;
}

extern "C" int pt_create(const pt_config* cfg, void* dev_weights, size_t weight_bytes, void* dev_kv,
                         size_t kv_bytes, void* dev_ws, size_t ws_bytes, void* hip_stream,
                         pt_handle** out) {
  int rc = pt_validate_config(cfg);
  if (rc) return rc;
  if (!out) return pt_set_error(PT_ERR_NULL_POINTER, "out is NULL");
  *out = nullptr;
  if (!dev_weights || !dev_kv || !dev_ws) return pt_set_error(PT_ERR_NULL_POINTER, "an arena pointer is NULL");
  if (((uintptr_t)dev_weights | (uintptr_t)dev_kv | (uintptr_t)dev_ws) & 255)
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "arena pointers must be 256-byte aligned");
  pt_layout l;
  pt_compute_layout(cfg, &l);
  if (weight_bytes < l.weight_bytes)
    return pt_set_error(PT_ERR_ARENA_TOO_SMALL, "weight arena: %zu bytes given, %zu needed", weight_bytes, l.weight_bytes);
  if (kv_bytes < l.kv_bytes)
    return pt_set_error(PT_ERR_ARENA_TOO_SMALL, "KV arena: %zu bytes given, %zu needed", kv_bytes, l.kv_bytes);
  if (ws_bytes < l.ws_bytes)
    return pt_set_error(PT_ERR_ARENA_TOO_SMALL, "workspace arena: %zu bytes given, %zu needed", ws_bytes, l.ws_bytes);
  pt_handle* h = new (std::nothrow) pt_handle();
  if (!h) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "out of host memory");
  h->cfg = *cfg;
  h->lay = l;
  h->w = (char*)dev_weights;
  h->kv = (char*)dev_kv;
  h->ws = (char*)dev_ws;
  pt_layout_workspace(cfg, &l, (int64_t)cfg->max_batch * l.s_k, cfg->max_batch, PT_SK_PART_FLOATS, PT_MAX_SPLITS, &h->arena);
  h->arena.base = h->ws;
  h->active = &h->arena;
  h->stream = (hipStream_t)hip_stream;
  h->batch = 0;
  h->seq_len = 0;
  h->ragged = false;
  h->merges = 0;
  h->weights_ready = false;
  h->rope_ready = false;
  h->taps = nullptr;
  h->track_taps = nullptr;
  h->routes_out = nullptr;
  h->routes_in = nullptr;
  h->path = PT_PATH_AUTO;
  *out = h;
  return PT_OK;
}

extern "C" int pt_destroy(pt_handle* h) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  for (const pt_prof_pair& p : h->prof.pending) { (void)hipEventDestroy(p.e0); (void)hipEventDestroy(p.e1); }
  for (hipEvent_t e : h->prof.free_events) (void)hipEventDestroy(e);
  delete h;
  return PT_OK;
}

extern "C" int pt_reset(pt_handle* h) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  h->batch = 0;
  h->seq_len = 0;
  h->ragged = false;
  h->seqs.clear();
  return PT_OK;
}

extern "C" int64_t pt_merge_count(const pt_handle* h) { return h ? h->merges : (int64_t)PT_ERR_NULL_POINTER; }
extern "C" int32_t pt_seq_len(const pt_handle* h) { return h ? h->seq_len : (int32_t)PT_ERR_NULL_POINTER; }

extern "C" int pt_set_taps(pt_handle* h, float* dev_taps, float* dev_track_taps) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  h->taps = dev_taps;
  h->track_taps = dev_track_taps;
  return PT_OK;
}

extern "C" int pt_set_moe_routes(pt_handle* h, int32_t* dev_routes_out, const int32_t* dev_routes_in) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (h->cfg.n_experts == 0) return pt_set_error(PT_ERR_BAD_STATE, "the model has no experts");
  h->routes_out = dev_routes_out;
  h->routes_in = dev_routes_in;
  return PT_OK;
}

extern "C" int pt_set_kernel_path(pt_handle* h, int32_t path) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (path != PT_PATH_AUTO && path != PT_PATH_GENERIC)
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown kernel path %d", path);
  h->path = path;
  return PT_OK;
}

extern "C" int pt_init_weights(pt_handle* h, uint64_t seed) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  int rc = pt_launch_weight_init(h, seed);
  if (rc) return rc;
  h->weights_ready = true;
  return PT_OK;
}

static int check_tensor(const pt_handle* h, int32_t tensor, int32_t track, int32_t layer) {
  if (tensor < PT_W_EMBED || tensor > PT_W_ROUTER) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown tensor id %d", tensor);
  const bool global = tensor == PT_W_EMBED || tensor == PT_W_HEAD || tensor == PT_W_GF;
  if (tensor == PT_W_ROUTER && h->cfg.n_experts == 0) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "the model has no router");
  if (h->cfg.n_experts > 0 && (tensor == PT_W_G || tensor == PT_W_U || tensor == PT_W_D)) {
    // per-expert tensors: layer = PT_EXPERT_LAYER(layer, expert)
    const int32_t expert = (layer >> 12) - 1;
    if (expert < 0 || expert >= h->cfg.n_experts)
      return pt_set_error(PT_ERR_INVALID_ARGUMENT, "expert tensors are addressed with layer = PT_EXPERT_LAYER(layer, expert); expert %d out of range", expert);
    layer &= 0xfff;
  }
  if ((tensor == PT_W_EMBED || tensor == PT_W_HEAD) && h->cfg.vocab == 0)
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "model has no vocabulary");
  if (!global && (track < 0 || track >= h->cfg.n_tracks || layer < 0 || layer >= h->cfg.n_layers))
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "track %d / layer %d out of range", track, layer);
  return PT_OK;
}

extern "C" int pt_set_weight(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, const float* dev_src) {
  if (!h || !dev_src) return pt_set_error(PT_ERR_NULL_POINTER, "handle or source is NULL");
  int rc = check_tensor(h, tensor, track, layer);
  if (rc) return rc;
  rc = pt_launch_weight_copy(h, tensor, track, layer, const_cast<float*>(dev_src), true);
  if (rc) return rc;
  h->weights_ready = true;
  return PT_OK;
}

extern "C" int pt_get_weight(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, float* dev_dst) {
  if (!h || !dev_dst) return pt_set_error(PT_ERR_NULL_POINTER, "handle or destination is NULL");
  int rc = check_tensor(h, tensor, track, layer);
  if (rc) return rc;
  return pt_launch_weight_copy(h, tensor, track, layer, dev_dst, false);
}

extern "C" int pt_track_merge(const void* const* host_tracks, int32_t n, int64_t tokens, int32_t d,
                              int32_t dtype, float scale, void* dev_out, void* hip_stream) {
  if (!host_tracks || !dev_out) return pt_set_error(PT_ERR_NULL_POINTER, "tracks or out is NULL");
  if (n < 1 || n > 16) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "n = %d, need 1..16", n);
  if (tokens < 0 || d < 8 || d % 8) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "tokens must be >= 0 and d a positive multiple of 8");
  if (dtype != PT_F32 && dtype != PT_BF16) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "dtype must be PT_F32 or PT_BF16");
  for (int i = 0; i < n; ++i) {
    if (!host_tracks[i]) return pt_set_error(PT_ERR_NULL_POINTER, "tracks[%d] is NULL", i);
    if ((uintptr_t)host_tracks[i] & 15) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "tracks[%d] is not 16-byte aligned", i);
  }
  if ((uintptr_t)dev_out & 15) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "out is not 16-byte aligned");
  if (tokens == 0) return PT_OK;
  return pt_launch_merge(host_tracks, n, tokens * d, dtype, scale, dev_out, nullptr, (hipStream_t)hip_stream);
}

extern "C" int pt_argmax(const float* dev_logits, int32_t rows, int32_t vocab, int32_t* dev_out, void* hip_stream) {
  if (!dev_logits || !dev_out) return pt_set_error(PT_ERR_NULL_POINTER, "logits or out is NULL");
  if (rows < 0 || vocab < 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "rows must be >= 0 and vocab >= 1");
  return pt_launch_argmax(dev_logits, rows, vocab, dev_out, (hipStream_t)hip_stream);
}

// ---------------------------------------------------------------------------------------------
// Per-kernel timing: a pair of events around each launch of a selected class.
// ---------------------------------------------------------------------------------------------
static hipEvent_t prof_get_event(pt_handle* h) {
  if (!h->prof.free_events.empty()) {
    hipEvent_t e = h->prof.free_events.back();
    h->prof.free_events.pop_back();
    return e;
  }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) return nullptr;
  return e;
}

struct prof_scope {
  pt_handle* h;
  int cls;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  prof_scope(pt_handle* h_, int cls_) : h(h_), cls(cls_) {
    if (h->prof.mask & (1u << cls)) {
      e0 = prof_get_event(h);
      e1 = prof_get_event(h);
      if (e0 && e1) (void)hipEventRecord(e0, h->stream);
    }
  }
  ~prof_scope() {
    if (e0 && e1) {
      (void)hipEventRecord(e1, h->stream);
      h->prof.pending.push_back({cls, e0, e1});
    }
  }
};

static int prof_fold(pt_handle* h) {
  if (h->prof.pending.empty()) return PT_OK;
  PT_HIP_CHECK(hipStreamSynchronize(h->stream));
  for (const pt_prof_pair& p : h->prof.pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.e0, p.e1) == hipSuccess) {
      h->prof.ms[p.cls] += ms;
      h->prof.launches[p.cls] += 1;
    }
    h->prof.free_events.push_back(p.e0);
    h->prof.free_events.push_back(p.e1);
  }
  h->prof.pending.clear();
  return PT_OK;
}

extern "C" int pt_profile_enable(pt_handle* h, uint32_t class_mask) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  h->prof.mask = class_mask & ((1u << PT_K_COUNT) - 1);
  return PT_OK;
}

extern "C" int pt_profile_read(pt_handle* h, int32_t kernel_class, double* total_ms, int64_t* launches) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (kernel_class < 0 || kernel_class >= PT_K_COUNT) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown kernel class %d", kernel_class);
  int rc = prof_fold(h);
  if (rc) return rc;
  if (total_ms) *total_ms = h->prof.ms[kernel_class];
  if (launches) *launches = h->prof.launches[kernel_class];
  return PT_OK;
}

extern "C" int pt_profile_reset(pt_handle* h) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  int rc = prof_fold(h);
  if (rc) return rc;
  for (int k = 0; k < PT_K_COUNT; ++k) {
    h->prof.ms[k] = 0;
    h->prof.launches[k] = 0;
    for (int f = 0; f < PT_FAMILY_COUNT; ++f) h->prof.family[k][f] = 0;
  }
  return PT_OK;
}

extern "C" int pt_profile_paths(pt_handle* h, int32_t kernel_class, int64_t* counts) {
  if (!h || !counts) return pt_set_error(PT_ERR_NULL_POINTER, "handle or counts is NULL");
  if (kernel_class < 0 || kernel_class >= PT_K_COUNT) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown kernel class %d", kernel_class);
  for (int f = 0; f < PT_FAMILY_COUNT; ++f) counts[f] = h->prof.family[kernel_class][f];
  return PT_OK;
}

extern "C" int pt_set_tuning(int32_t knob, int32_t value) {
  if (knob == PT_TUNE_GEMM_TILE_CONFIG) pt_tune_gemm_cfg = value;
  else if (knob == PT_TUNE_SKINNY_PLAN) pt_tune_skinny_plan = value;
  else if (knob == PT_TUNE_FOLD_RMSNORM) g_fold_rmsnorm = value != 0;
  else if (knob == PT_TUNE_ATTN_PREFILL) pt_tune_attn_prefill = value != 0;
  else return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown tuning knob %d", knob);
  return PT_OK;
}

extern "C" int pt_sync_status(pt_handle* h) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (!h->rope_ready) {   // no forward call yet: nothing can have raised the flag
    PT_HIP_CHECK(hipStreamSynchronize(h->stream));
    return PT_OK;
  }
  int32_t flag = 0;
  int32_t* dev_flag = (int32_t*)(h->w + h->lay.off_flag);
  PT_HIP_CHECK(hipMemcpyAsync(&flag, dev_flag, sizeof(flag), hipMemcpyDeviceToHost, h->stream));
  PT_HIP_CHECK(hipStreamSynchronize(h->stream));
  if (flag) {
    int rc = pt_launch_fill_f32((float*)dev_flag, 1, 0.0f, h->stream);   // all-zero bits
    if (rc) return rc;
    if (flag & 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "a token id outside [0, vocab) was given to a forward call");
    if (flag & 2) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "a prescribed expert selection held an expert out of range or twice");
  }
  return PT_OK;
}

// ---------------------------------------------------------------------------------------------
// The forward pass.  rows = B*S rows per track; row m is sequence m / S at position pos0 + m % S.
// ---------------------------------------------------------------------------------------------
// Records which kernel family served a launch of class cls (pt_profile_paths).
static inline void count_family(pt_handle* h, int cls, int family) {
  if (family >= 0 && family < PT_FAMILY_COUNT) h->prof.family[cls][family] += 1;
}

static int run_gemm(pt_handle* h, const pt_gemm_args& g_in, int cls) {
  prof_scope ps(h, cls);
  pt_gemm_args g = g_in;
  g.sk_part = (float*)(h->active->base + h->active->off_skp);
  g.sk_part_floats = h->active->skp_floats;
  if (h->path == PT_PATH_AUTO) {
    int r = g.M <= 64 || g.n_groups > 0 ? pt_launch_gemm_skinny(g, false, h->stream) : 0;
    if (r < 0) return r;
    if (r > 0) { count_family(h, cls, r); return PT_OK; }
    if (g.norm_src) return pt_set_error(PT_ERR_HIP, "a GEMM that was to form its own normalised operand was not taken by that kernel");
    r = pt_launch_gemm_mfma(g, h->stream);
    if (r < 0) return r;
    if (r > 0) { count_family(h, cls, r); return PT_OK; }
  }
  count_family(h, cls, PT_FAMILY_GENERIC);
  return pt_launch_gemm_generic(g, h->stream);
}

// Residual GEMM (out = res + A W^T) followed, when gain is given, by the RMSNorm of the new residual stream
// into `normed`.  In decode the GEMM may split K over workgroups; the kernel that adds the slices also adds the
// residual and normalises.
//
// Prefill (more than 64 rows, MFMA tile kernels on both sides): the norm is folded into the two GEMMs instead.
// The residual GEMM's epilogue also stores bf16(h * gain) into `normed` and per-row partial sums of squares;
// the GEMM that consumes `normed` (`next`: its shape) multiplies its accumulators by the row's 1/rms.
// A small kernel turns the partial sums into one factor per row.  *folded_parts > 0 tells the caller that
// `normed` is unnormalised and the consumer must apply those factors (0: `normed` holds the finished RMSNorm).
static int run_residual_gemm_norm(pt_handle* h, const pt_gemm_args& g_in, int cls, const float* gain,
                                  int64_t gain_bstride, void* normed, const pt_gemm_args* next, int* folded_parts) {
  const pt_config& c = h->cfg;
  pt_gemm_args g = g_in;
  g.sk_part = (float*)(h->active->base + h->active->off_skp);
  g.sk_part_floats = h->active->skp_floats;
  const int64_t rows = g.M;
  int rc;
  *folded_parts = 0;
  if (h->path == PT_PATH_AUTO && g_fold_rmsnorm && gain && next && g.M > 64 && g.N == g.ldo && pt_gemm_mfma_covers(*next)) {
    const int parts = pt_gemm_mfma_fold_parts(g);
    if (parts > 0 && parts <= (g.N + 63) / 64) {
      g.nf_out = normed; g.nf_out_bstride = rows * g.N;
      g.nf_gain = gain; g.nf_gain_bstride = gain_bstride;
      g.nf_ss = (float*)(h->active->base + h->active->off_ss); g.nf_ss_bstride = rows * parts;
      g.nf_parts = parts;
      rc = run_gemm(h, g, cls);
      if (rc) return rc;
      *folded_parts = parts;
      prof_scope ps(h, PT_K_RMSNORM);
      return pt_launch_row_inv_rms(g.nf_ss, parts, (int64_t)g.batch * rows, g.N, c.rms_eps,
                                   (float*)(h->active->base + h->active->off_rinv), h->stream);
    }
  }
  if (h->path == PT_PATH_AUTO && g.M <= 64 && g.N == g.ldo && g.N <= 8192 && pt_gemm_skinny_ksplit(g) > 1) {
    const int slices = pt_gemm_skinny_ksplit(g);
    {
      prof_scope ps(h, cls);
      rc = pt_launch_gemm_skinny(g, true, h->stream);
      if (rc < 0) return rc;
      if (rc == 0) return pt_set_error(PT_ERR_HIP, "decode GEMM refused a shape it had accepted");
      count_family(h, cls, rc);
    }
    prof_scope ps(h, PT_K_RMSNORM);
    return pt_launch_resnorm(g.sk_part, slices, g.res, g.res_bstride, g.out, g.out_bstride, gain, gain_bstride,
                             gain ? normed : nullptr, rows * g.N, g.batch, rows, g.N, c.rms_eps, h->stream);
  }
  rc = run_gemm(h, g_in, cls);
  if (rc || !gain) return rc;
  prof_scope ps(h, PT_K_RMSNORM);
  return pt_launch_rmsnorm(g.out, g.out_bstride, gain, gain_bstride, normed, rows * g.N, c.dtype, g.batch, rows,
                           g.N, c.rms_eps, h->stream);
}

static int run_attention(pt_handle* h, const pt_attn_args& a) {
  const int cls = a.S == 1 ? PT_K_ATTN_DECODE : PT_K_ATTN_PREFILL;
  prof_scope ps(h, cls);
  if (h->path == PT_PATH_AUTO) {
    int r = a.S == 1 ? pt_launch_attn_decode(a, h->stream) : pt_launch_attn_prefill_mfma(a, h->stream);
    if (r < 0) return r;
    if (r > 0) { count_family(h, cls, r); return PT_OK; }
  }
  count_family(h, cls, PT_FAMILY_GENERIC);
  return pt_launch_attn_generic(a, h->stream);
}

// A ragged batch as the forward pass sees it (device pointers).  Prefill: the padded-packed row layout
// (seq_info, row_map over `rows` packed rows, `valid`: packed row of every real token in input order, `last`:
// packed row of each sequence's last token).  Decode: row_map[b] = (b, length of b) only.
struct ragged_ctx {
  const int4* seq_info;
  const int2* row_map;
  const int32_t* valid;
  const int32_t* last;
  int64_t rows, n_valid;
  int32_t max_plen, max_pos;
};

static int forward(pt_handle* h, const pt_workspace& w, const int32_t* dev_tokens, const float* dev_hidden_in,
                   int32_t hidden_tracks, int32_t B, int32_t S, int32_t pos0, int32_t logits_mode,
                   float* dev_logits, float* dev_hidden_out, int32_t* dev_argmax, const ragged_ctx* rg = nullptr) {
  h->active = &w;
  const bool ragged_prefill = rg && S != 1;
  const pt_config& c = h->cfg;
  const pt_layout& l = h->lay;
  const int64_t T = c.n_tracks, L = c.n_layers, d = c.d_model, f = c.d_ffn;
  const int64_t rows = ragged_prefill ? rg->rows : (int64_t)B * S;
  const int64_t es = l.elem_size;
  hipStream_t st = h->stream;
  int rc;

  if (!h->rope_ready) {
    rc = pt_launch_rope_table((float*)(h->w + l.off_rope), (int32_t)l.s_k, c.head_dim, c.rope_theta, st);
    if (rc) return rc;
    rc = pt_launch_fill_f32((float*)(h->w + l.off_flag), 1, 0.0f, st);   // device status word: all-zero bits
    if (rc) return rc;
    h->rope_ready = true;
  }

  float* hres = (float*)(w.base + w.off_h);   // [T, rows, d]
  float* hm = (float*)(w.base + w.off_hm);    // [rows, d]
  const float* merged = hm;                  // the output activation of Algorithm 1 after the last merge
  char* abuf = w.base + w.off_a;
  char* qbuf = w.base + w.off_q;
  char* obuf = w.base + w.off_o;
  char* mbuf = w.base + w.off_m;
  const float* gains = (const float*)(h->w + l.off_gains);

  // Algorithm 1, first line: every track starts from the same embedding input x.  x is kept
  // once; the first layer of a block reads it with a zero track stride.
  const float* x;
  int64_t x_bstride;
  if (dev_hidden_in && ragged_prefill) {
    // the caller's rows are packed without padding: spread them over the padded rows (zeros in between).  Per-track
    // inputs go to the residual buffer, which the first layer reads and then overwrites element by element.
    float* xp = hidden_tracks == 1 ? hm : hres;
    rc = pt_launch_scatter_rows(dev_hidden_in, hidden_tracks == 1 ? 0 : rg->n_valid * d, rg->row_map, rg->seq_info, rows,
                                (int32_t)d, hidden_tracks, xp, rows * d, st);
    if (rc) return rc;
    x = xp;
    x_bstride = hidden_tracks == 1 ? 0 : rows * d;
  } else if (dev_hidden_in) {
    x = dev_hidden_in;
    x_bstride = hidden_tracks == 1 ? 0 : rows * d;
  } else if (ragged_prefill) {
    { prof_scope ps(h, PT_K_EMBED); rc = pt_launch_embed_ragged(h->w + l.off_embed, c.dtype, dev_tokens, rg->row_map, rg->seq_info, rows, (int32_t)d, c.vocab, hm, (int32_t*)(h->w + l.off_flag), st); }
    if (rc) return rc;
    x = hm;
    x_bstride = 0;
  } else {
    { prof_scope ps(h, PT_K_EMBED); rc = pt_launch_embed(h->w + l.off_embed, c.dtype, dev_tokens, rows, (int32_t)d, c.vocab, hm, (int32_t*)(h->w + l.off_flag), st); }
    if (rc) return rc;
    x = hm;
    x_bstride = 0;
  }

  const int64_t kv_head_k = l.s_k * c.head_dim;
  const int64_t kv_head_v = (int64_t)c.head_dim * l.s_pad;
  int merge_idx = 0;
  bool normed = false;   // abuf already holds the normalised input of this layer's attention half
  // Latency-mode decode (a handful of rows): the QKV and gate/up kernels form their RMSNorm-ed operand
  // themselves, which saves two launches per layer.  The decision depends on shapes only.
  bool fuse_qkv_norm = false, fuse_ffn_norm = false;
  pt_gemm_args qkv_proto, gu_proto;   // shapes of the two GEMMs that consume a normalised activation
  memset(&qkv_proto, 0, sizeof(qkv_proto));
  memset(&gu_proto, 0, sizeof(gu_proto));
  int qkv_rs_parts = 0;   // > 0: abuf holds bf16(h * gain) and the QKV GEMM applies the row scale (folded RMSNorm)
  if (h->path == PT_PATH_AUTO) {
    pt_gemm_args p;
    memset(&p, 0, sizeof(p));
    p.A = abuf; p.W = h->w + l.off_layers; p.lda = p.ldb = p.K = (int32_t)d;
    p.a_bstride = rows * d; p.w_bstride = L * l.layer_w_elems;
    p.M = (int32_t)rows; p.batch = (int32_t)T; p.dtype = c.dtype;
    p.N = (int32_t)l.n_qkv; p.epi = EPI_QKV; p.olp = qbuf; p.olp_bstride = rows * l.hq;
    p.H = c.n_heads; p.Hkv = c.n_kv_heads; p.hd = c.head_dim; p.S = S; p.s_pad = (int32_t)l.s_pad;
    p.row_map = rg ? rg->row_map : nullptr; p.row_blocks = ragged_prefill;
    fuse_qkv_norm = pt_gemm_fuses_norm(p);
    qkv_proto = p;
    p.N = (int32_t)(2 * f); p.epi = EPI_SWIGLU; p.olp = mbuf; p.olp_bstride = rows * f;
    fuse_ffn_norm = pt_gemm_fuses_norm(p) && c.n_experts == 0;
    gu_proto = p;
  }
  // PT-MoE: the feed-forward half of every layer is a routed mixture of experts (moe_ffn below); the RMSNorm in
  // front of it is always materialised, because the router and the gathered expert GEMMs both read it
  const bool moe = c.n_experts > 0;
  pt_moe_args ma;
  int64_t moe_nblk = 0;
  memset(&ma, 0, sizeof(ma));
  if (moe) {
    ma.T = (int32_t)T; ma.E = c.n_experts; ma.e_pad = (int32_t)l.e_pad; ma.k = c.top_k;
    // slots of this call's rows (the workspace was laid out for at least as many)
    ma.rows = rows; ma.slots = (rows * c.top_k + (int64_t)c.n_experts * 255 + 255) / 256 * 256;
    if (ma.slots > w.slots) return pt_set_error(PT_ERR_CAPACITY, "expert slots exceed the workspace");
    moe_nblk = (rows + 255) / 256;   // counting blocks of 256 rows: the layout of ma.cnt
    ma.logits = (const float*)(w.base + w.off_rlogit);
    ma.route = (int32_t*)(w.base + w.off_route);
    ma.gate = (float*)(w.base + w.off_gate);
    ma.slot = (int32_t*)(w.base + w.off_slot);
    ma.perm = (int32_t*)(w.base + w.off_perm);
    ma.blk = (int32_t*)(w.base + w.off_blk);
    ma.cnt = (int32_t*)(w.base + w.off_cnt);
    ma.obs_bstride = rows * c.top_k;
    ma.flag = (int32_t*)(h->w + l.off_flag);
  }
  for (int64_t layer = 0; layer < L; ++layer) {
    const bool first = (layer % c.block_depth) == 0;
    const float* src = first ? x : hres;
    const int64_t src_bstride = first ? x_bstride : rows * d;
    const char* wl = h->w + l.off_layers + (size_t)(layer * l.layer_w_elems * es);
    const int64_t w_bstride = L * l.layer_w_elems;

    // attention half
    if (!normed && !fuse_qkv_norm) {
      prof_scope ps(h, PT_K_RMSNORM);
      rc = pt_launch_rmsnorm(src, src_bstride, gains + (layer * 2 + 0) * d, L * 2 * d, abuf, rows * d,
                             c.dtype, (int32_t)T, rows, (int32_t)d, c.rms_eps, st);
      if (rc) return rc;
    }
    pt_gemm_args g;
    memset(&g, 0, sizeof(g));
    g.A = abuf; g.a_bstride = rows * d; g.lda = (int32_t)d;
    g.W = wl; g.w_bstride = w_bstride; g.ldb = (int32_t)d;
    g.M = (int32_t)rows; g.N = (int32_t)l.n_qkv; g.K = (int32_t)d; g.batch = (int32_t)T;
    g.dtype = c.dtype; g.epi = EPI_QKV;
    g.olp = qbuf; g.olp_bstride = rows * l.hq;
    g.kc = h->kv + l.off_k + (size_t)(layer * c.max_batch * c.n_kv_heads * kv_head_k * es);
    g.vc = h->kv + l.off_v + (size_t)(layer * c.max_batch * c.n_kv_heads * kv_head_v * es);
    g.rope = (const float*)(h->w + l.off_rope);
    g.H = c.n_heads; g.Hkv = c.n_kv_heads; g.hd = c.head_dim; g.S = S; g.pos0 = pos0;
    g.s_pad = (int32_t)l.s_pad;
    g.row_map = rg ? rg->row_map : nullptr; g.row_blocks = ragged_prefill;
    // cache strides are stated for K; the V^T side uses hd * s_pad per head with the same nesting
    g.kv_bstride = L * c.max_batch * c.n_kv_heads;   // in heads; kernels scale by the head size
    g.kv_seq_stride = c.n_kv_heads;                  // in heads
    g.kv_head_elems = kv_head_k;
    if (fuse_qkv_norm) {
      g.norm_src = src; g.norm_bstride = src_bstride;
      g.norm_gain = gains + (layer * 2 + 0) * d; g.norm_gbstride = L * 2 * d; g.norm_eps = c.rms_eps;
    }
    if (qkv_rs_parts > 0) {
      g.rs_inv = (const float*)(w.base + w.off_rinv); g.rs_bstride = rows;
    }
    rc = run_gemm(h, g, PT_K_GEMM_QKV);
    if (rc) return rc;

    pt_attn_args a;
    memset(&a, 0, sizeof(a));
    a.q = qbuf; a.o = obuf; a.kc = g.kc; a.vc = g.vc;
    a.q_bstride = rows * l.hq;
    a.kv_bstride = g.kv_bstride; a.kv_seq_stride = g.kv_seq_stride; a.kv_head_elems = kv_head_k;
    a.n_tracks = (int32_t)T; a.B = B; a.S = S; a.pos0 = pos0;
    a.H = c.n_heads; a.Hkv = c.n_kv_heads; a.hd = c.head_dim; a.s_pad = (int32_t)l.s_pad;
    a.dtype = c.dtype;
    a.partials = (float*)(w.base + w.off_part); a.max_splits = w.max_splits;
    if (rg) {
      a.row_map = rg->row_map; a.seq_info = ragged_prefill ? rg->seq_info : nullptr;
      a.max_pos = rg->max_pos; a.max_plen = rg->max_plen; a.rows = rows;
    }
    rc = run_attention(h, a);
    if (rc) return rc;

    memset(&g, 0, sizeof(g));
    g.A = obuf; g.a_bstride = rows * l.hq; g.lda = (int32_t)l.hq;
    g.W = wl + (size_t)(l.wqkv_elems * es); g.w_bstride = w_bstride; g.ldb = (int32_t)l.hq;
    g.M = (int32_t)rows; g.N = (int32_t)d; g.K = (int32_t)l.hq; g.batch = (int32_t)T;
    g.dtype = c.dtype; g.epi = EPI_RESIDUAL;
    g.out = hres; g.out_bstride = rows * d; g.ldo = (int32_t)d;
    g.res = src; g.res_bstride = src_bstride;
    // ... and the RMSNorm that opens the feed-forward half
    int gu_rs_parts = 0;
    rc = run_residual_gemm_norm(h, g, PT_K_GEMM_OUT, fuse_ffn_norm ? nullptr : gains + (layer * 2 + 1) * d, L * 2 * d, abuf,
                                moe ? nullptr : &gu_proto, &gu_rs_parts);
    if (rc) return rc;

    // inside a block the next layer's first RMSNorm follows directly; at a block end the merge comes first
    const bool block_end = (layer + 1) % c.block_depth == 0;
    const bool norm_next = !block_end && !fuse_qkv_norm;

    if (moe) {
      // feed-forward half, PT-MoE: router logits -> expert selection and grouping -> gate/up and down GEMMs over the
      // slots of every expert -> gate-weighted sum into the residual stream (and the next RMSNorm)
      const char* wexp = wl + (size_t)(l.off_exp_elems * es);
      memset(&g, 0, sizeof(g));
      g.A = abuf; g.a_bstride = rows * d; g.lda = (int32_t)d;
      g.W = wl + (size_t)(l.off_wr_elems * es); g.w_bstride = w_bstride; g.ldb = (int32_t)d;
      g.M = (int32_t)rows; g.N = (int32_t)l.e_pad; g.K = (int32_t)d; g.batch = (int32_t)T;
      g.dtype = c.dtype; g.epi = EPI_STORE_F32;
      g.out = (float*)(w.base + w.off_rlogit); g.out_bstride = rows * l.e_pad; g.ldo = (int32_t)l.e_pad;
      rc = run_gemm(h, g, PT_K_GEMM_ROUTER);
      if (rc) return rc;
      {
        prof_scope ps(h, PT_K_MOE);
        const int64_t obs = layer * T * rows * c.top_k;
        ma.forced = h->routes_in ? h->routes_in + obs : nullptr;
        ma.chosen_out = h->routes_out ? h->routes_out + obs : nullptr;
        rc = pt_launch_moe_route(ma, st);
      }
      if (rc) return rc;
      memset(&g, 0, sizeof(g));
      g.A = abuf; g.a_bstride = rows * d; g.lda = (int32_t)d;
      g.a_rows = ma.perm; g.a_rows_bstride = ma.slots;
      g.blk_group = ma.blk; g.grp_bstride = ma.slots / 64; g.w_gstride = l.expert_elems;
      g.grp_rows = (int32_t)((rows * c.top_k + c.n_experts - 1) / c.n_experts);
      g.grp_count = ma.cnt + moe_nblk * 64; g.grp_base = ma.cnt + (moe_nblk + 1) * 64; g.grp_info_bstride = (moe_nblk + 2) * 64;
      g.n_groups = c.n_experts; g.grp_max_rows = (int32_t)std::min<int64_t>(rows, 0x7fffffff);
      g.W = wexp; g.w_bstride = w_bstride; g.ldb = (int32_t)d;
      g.M = (int32_t)ma.slots; g.N = (int32_t)(2 * f); g.K = (int32_t)d; g.batch = (int32_t)T;
      g.dtype = c.dtype; g.epi = EPI_SWIGLU;
      g.olp = mbuf; g.olp_bstride = ma.slots * f;
      rc = run_gemm(h, g, PT_K_GEMM_GATEUP);
      if (rc) return rc;
      float* ybuf = (float*)(w.base + w.off_y);
      memset(&g, 0, sizeof(g));
      g.A = mbuf; g.a_bstride = ma.slots * f; g.lda = (int32_t)f;
      g.blk_group = ma.blk; g.grp_bstride = ma.slots / 64; g.w_gstride = l.expert_elems;
      g.grp_rows = (int32_t)((rows * c.top_k + c.n_experts - 1) / c.n_experts);
      g.grp_count = ma.cnt + moe_nblk * 64; g.grp_base = ma.cnt + (moe_nblk + 1) * 64; g.grp_info_bstride = (moe_nblk + 2) * 64;
      g.n_groups = c.n_experts; g.grp_max_rows = (int32_t)std::min<int64_t>(rows, 0x7fffffff);
      g.W = wexp + (size_t)(l.wgu_elems * es); g.w_bstride = w_bstride; g.ldb = (int32_t)f;
      g.M = (int32_t)ma.slots; g.N = (int32_t)d; g.K = (int32_t)f; g.batch = (int32_t)T;
      g.dtype = c.dtype; g.epi = EPI_STORE_F32;
      g.out = ybuf; g.out_bstride = ma.slots * d; g.ldo = (int32_t)d;
      rc = run_gemm(h, g, PT_K_GEMM_DOWN);
      if (rc) return rc;
      {
        prof_scope ps(h, PT_K_MOE);
        rc = pt_launch_moe_combine(ma, ybuf, hres, rows * d, hres, (int32_t)d,
                                   norm_next ? gains + ((layer + 1) * 2 + 0) * d : nullptr, L * 2 * d,
                                   norm_next ? abuf : nullptr, c.dtype, c.rms_eps, st);
      }
      if (rc) return rc;
      qkv_rs_parts = 0;
    } else {
    // feed-forward half
    memset(&g, 0, sizeof(g));
    g.A = abuf; g.a_bstride = rows * d; g.lda = (int32_t)d;
    g.W = wl + (size_t)((l.wqkv_elems + l.wo_elems) * es); g.w_bstride = w_bstride; g.ldb = (int32_t)d;
    g.M = (int32_t)rows; g.N = (int32_t)(2 * f); g.K = (int32_t)d; g.batch = (int32_t)T;
    g.dtype = c.dtype; g.epi = EPI_SWIGLU;
    g.olp = mbuf; g.olp_bstride = rows * f;
    if (fuse_ffn_norm) {
      g.norm_src = hres; g.norm_bstride = rows * d;
      g.norm_gain = gains + (layer * 2 + 1) * d; g.norm_gbstride = L * 2 * d; g.norm_eps = c.rms_eps;
    }
    if (gu_rs_parts > 0) {
      g.rs_inv = (const float*)(w.base + w.off_rinv); g.rs_bstride = rows;
    }
    rc = run_gemm(h, g, PT_K_GEMM_GATEUP);
    if (rc) return rc;
    memset(&g, 0, sizeof(g));
    g.A = mbuf; g.a_bstride = rows * f; g.lda = (int32_t)f;
    g.W = wl + (size_t)((l.wqkv_elems + l.wo_elems + l.wgu_elems) * es); g.w_bstride = w_bstride; g.ldb = (int32_t)f;
    g.M = (int32_t)rows; g.N = (int32_t)d; g.K = (int32_t)f; g.batch = (int32_t)T;
    g.dtype = c.dtype; g.epi = EPI_RESIDUAL;
    g.out = hres; g.out_bstride = rows * d; g.ldo = (int32_t)d;
    g.res = hres; g.res_bstride = rows * d;
    rc = run_residual_gemm_norm(h, g, PT_K_GEMM_DOWN, norm_next ? gains + ((layer + 1) * 2 + 0) * d : nullptr,
                                L * 2 * d, abuf, &qkv_proto, &qkv_rs_parts);
    if (rc) return rc;
    }
    normed = norm_next;

    // Algorithm 1: after every D-th layer, all-reduce the track activations; every track
    // continues from the reduced activation.
    if ((layer + 1) % c.block_depth == 0) {
      const void* tr[16];
      for (int64_t t = 0; t < T; ++t) tr[t] = hres + t * rows * d;
      // observation points: all rows, or (ragged prefill) the rows of the real tokens in input order
      const int64_t tap_rows = ragged_prefill ? rg->n_valid : rows;
      if (h->track_taps) {
        float* tt = h->track_taps + (int64_t)merge_idx * T * tap_rows * d;
        if (ragged_prefill) {
          for (int64_t t = 0; t < T && !rc; ++t) rc = pt_launch_gather_rows(hres + t * rows * d, rg->valid, tap_rows, (int32_t)d, tt + t * tap_rows * d, st);
        } else {
          rc = pt_launch_copy_f32(hres, tt, T * rows * d, st);
        }
        if (rc) return rc;
      }
      float* tap = h->taps ? h->taps + (int64_t)merge_idx * tap_rows * d : nullptr;
      float* tap_gather = nullptr;
      if (ragged_prefill && tap) { tap_gather = tap; tap = nullptr; }
      if (T == 1 && c.merge_scale == 1.0f && !tap && !tap_gather) {
        // one track, plain sum: the all-reduce is the identity and the track simply continues
        merged = hres;
        x = hres;
        x_bstride = rows * d;
      } else {
        {
          prof_scope ps(h, PT_K_MERGE);
          rc = pt_launch_merge(tr, (int32_t)T, rows * d, PT_F32, c.merge_scale, hm, tap, st);
        }
        if (rc) return rc;
        if (tap_gather) {
          rc = pt_launch_gather_rows(hm, rg->valid, tap_rows, (int32_t)d, tap_gather, st);
          if (rc) return rc;
        }
        merged = hm;
        x = hm;
        x_bstride = 0;
      }
      ++merge_idx;
      ++h->merges;
    }
  }

  if (dev_hidden_out) {
    rc = ragged_prefill ? pt_launch_gather_rows(merged, rg->valid, rg->n_valid, (int32_t)d, dev_hidden_out, st)
                        : pt_launch_copy_f32(merged, dev_hidden_out, rows * d, st);
    if (rc) return rc;
  }
  if (logits_mode != PT_LOGITS_NONE && (dev_logits || dev_argmax)) {
    const int64_t lrows = logits_mode == PT_LOGITS_ALL ? (ragged_prefill ? rg->n_valid : rows) : B;
    const float* gf = (const float*)(h->w + l.off_gf);
    if (ragged_prefill)   // the rows of the real tokens (all of them, or each sequence's last one), gathered by index
      rc = pt_launch_rmsnorm_rows(merged, gf, abuf, c.dtype, lrows, 0, 0, logits_mode == PT_LOGITS_ALL ? rg->valid : rg->last,
                                  (int32_t)d, c.rms_eps, st);
    else if (logits_mode == PT_LOGITS_ALL)
      rc = pt_launch_rmsnorm_rows(merged, gf, abuf, c.dtype, lrows, 1, 0, nullptr, (int32_t)d, c.rms_eps, st);
    else
      rc = pt_launch_rmsnorm_rows(merged, gf, abuf, c.dtype, lrows, S, S - 1, nullptr, (int32_t)d, c.rms_eps, st);
    if (rc) return rc;
    float* lg = dev_logits;
    if (!lg) return pt_set_error(PT_ERR_NULL_POINTER, "argmax needs a logits buffer");
    pt_gemm_args g;
    memset(&g, 0, sizeof(g));
    g.A = abuf; g.a_bstride = 0; g.lda = (int32_t)d;
    g.W = h->w + l.off_headT; g.w_bstride = 0; g.ldb = (int32_t)d;
    g.M = (int32_t)lrows; g.N = c.vocab; g.K = (int32_t)d; g.batch = 1;
    g.dtype = c.dtype; g.epi = EPI_STORE_F32;
    g.out = lg; g.out_bstride = 0; g.ldo = c.vocab;
    rc = run_gemm(h, g, PT_K_GEMM_HEAD);
    if (rc) return rc;
    if (dev_argmax) {
      rc = pt_launch_argmax(lg, (int32_t)lrows, c.vocab, dev_argmax, st);
      if (rc) return rc;
    }
  }
  return PT_OK;
}

static int check_inputs(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                        int32_t hidden_tracks) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (!h->weights_ready) return pt_set_error(PT_ERR_BAD_STATE, "weights have not been initialised");
  if (!dev_tokens && !dev_hidden_in) return pt_set_error(PT_ERR_NULL_POINTER, "neither tokens nor hidden input given");
  if (!dev_hidden_in && h->cfg.vocab == 0) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "model has no vocabulary: pass hidden states");
  if (dev_hidden_in && hidden_tracks != 1 && hidden_tracks != h->cfg.n_tracks)
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "hidden_tracks = %d, need 1 or n_tracks", hidden_tracks);
  return PT_OK;
}

extern "C" int pt_prefill(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                          int32_t hidden_tracks, int32_t B, int32_t S, int32_t logits_mode,
                          float* dev_logits, float* dev_hidden_out) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (B < 1 || S < 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "B and S must be >= 1");
  if (B > h->cfg.max_batch) return pt_set_error(PT_ERR_CAPACITY, "B = %d exceeds max_batch = %d", B, h->cfg.max_batch);
  if (S > h->cfg.max_seq) return pt_set_error(PT_ERR_CAPACITY, "S = %d exceeds max_seq = %d", S, h->cfg.max_seq);
  if (logits_mode < PT_LOGITS_NONE || logits_mode > PT_LOGITS_ALL) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "bad logits_mode");
  if (logits_mode != PT_LOGITS_NONE) {
    if (h->cfg.vocab == 0) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "model has no vocabulary: no logits");
    if (!dev_logits) return pt_set_error(PT_ERR_NULL_POINTER, "logits requested but dev_logits is NULL");
  }
  int rc = check_inputs(h, dev_tokens, dev_hidden_in, hidden_tracks);
  if (rc) return rc;
  rc = forward(h, h->arena, dev_tokens, dev_hidden_in, hidden_tracks, B, S, 0, logits_mode, dev_logits, dev_hidden_out, nullptr);
  h->active = &h->arena;
  if (rc) return rc;
  h->batch = B;
  h->seq_len = S;
  h->ragged = false;
  h->seqs.clear();
  return PT_OK;
}

extern "C" int pt_prefill_ragged(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                                 int32_t hidden_tracks, int32_t B, const int32_t* host_lens, int32_t logits_mode,
                                 float* dev_logits, float* dev_hidden_out) {
  if (!h) return pt_set_error(PT_ERR_NULL_POINTER, "handle is NULL");
  if (!host_lens) return pt_set_error(PT_ERR_NULL_POINTER, "host_lens is NULL");
  if (B < 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "B must be >= 1");
  if (B > h->cfg.max_batch) return pt_set_error(PT_ERR_CAPACITY, "B = %d exceeds max_batch = %d", B, h->cfg.max_batch);
  if (logits_mode < PT_LOGITS_NONE || logits_mode > PT_LOGITS_ALL) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "bad logits_mode");
  if (logits_mode != PT_LOGITS_NONE) {
    if (h->cfg.vocab == 0) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "model has no vocabulary: no logits");
    if (!dev_logits) return pt_set_error(PT_ERR_NULL_POINTER, "logits requested but dev_logits is NULL");
  }
  if (h->routes_out || h->routes_in)
    return pt_set_error(PT_ERR_BAD_STATE, "the expert-selection observation points (pt_set_moe_routes) are not available for a ragged prefill");
  int rc = check_inputs(h, dev_tokens, dev_hidden_in, hidden_tracks);
  if (rc) return rc;
  // padded-packed layout: every sequence starts on a multiple of 64 rows
  std::vector<pt_seq> seqs((size_t)B);
  int64_t rows = 0, n_valid = 0;
  int32_t max_len = 0;
  for (int b = 0; b < B; ++b) {
    const int32_t len = host_lens[b];
    if (len < 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "host_lens[%d] = %d, need >= 1", b, len);
    if (len > h->cfg.max_seq) return pt_set_error(PT_ERR_CAPACITY, "host_lens[%d] = %d exceeds max_seq = %d", b, len, h->cfg.max_seq);
    const int32_t plen = (len + 63) / 64 * 64;
    if (rows + plen > 0x7fffffff || n_valid + len > 0x7fffffff) return pt_set_error(PT_ERR_CAPACITY, "batch too large");
    seqs[b] = {(int32_t)rows, plen, len, (int32_t)n_valid};
    rows += plen;
    n_valid += len;
    if (len > max_len) max_len = len;
  }
  h->seqs.swap(seqs);
  const pt_workspace& w = h->arena;
  int4* seq_info = (int4*)(h->kv + h->lay.off_seq);
  PT_HIP_CHECK(hipMemcpyAsync(seq_info, h->seqs.data(), (size_t)B * sizeof(pt_seq), hipMemcpyHostToDevice, h->stream));
  int2* row_map = (int2*)(w.base + w.off_rowmap);
  int32_t* last = (int32_t*)(w.base + w.off_rowidx);
  int32_t* valid = last + h->cfg.max_batch;
  rc = pt_launch_ragged_maps(seq_info, B, rows, row_map, valid, last, h->stream);
  if (rc) return rc;
  ragged_ctx rg;
  rg.seq_info = seq_info; rg.row_map = row_map; rg.valid = valid; rg.last = last;
  rg.rows = rows; rg.n_valid = n_valid;
  rg.max_plen = (max_len + 63) / 64 * 64; rg.max_pos = max_len - 1;
  rc = forward(h, w, dev_tokens, dev_hidden_in, hidden_tracks, B, rg.max_plen, 0, logits_mode, dev_logits, dev_hidden_out,
               nullptr, &rg);
  h->active = &h->arena;
  if (rc) { h->batch = 0; h->ragged = false; return rc; }
  h->batch = B;
  h->seq_len = max_len;
  h->ragged = true;
  return PT_OK;
}

extern "C" int pt_seq_lens(const pt_handle* h, int32_t* host_out) {
  if (!h || !host_out) return pt_set_error(PT_ERR_NULL_POINTER, "handle or out is NULL");
  for (int b = 0; b < h->batch; ++b) host_out[b] = h->ragged ? h->seqs[(size_t)b].len : h->seq_len;
  return PT_OK;
}

static int decode_checks(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in, int32_t hidden_tracks,
                         int32_t B, const float* dev_logits, const int32_t* dev_argmax) {
  int rc = check_inputs(h, dev_tokens, dev_hidden_in, hidden_tracks);
  if (rc) return rc;
  if (h->batch == 0) return pt_set_error(PT_ERR_BAD_STATE, "decode before prefill");
  if (B != h->batch) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "B = %d differs from the prefilled batch %d", B, h->batch);
  if (h->seq_len + 1 > h->cfg.max_seq) return pt_set_error(PT_ERR_CAPACITY, "sequence length %d + 1 exceeds max_seq = %d", h->seq_len, h->cfg.max_seq);
  if ((dev_logits || dev_argmax) && h->cfg.vocab == 0) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "model has no vocabulary: no logits");
  if (dev_argmax && !dev_logits) return pt_set_error(PT_ERR_NULL_POINTER, "argmax needs a logits buffer");
  return PT_OK;
}

// One decode step over the temporaries `w`.  A ragged batch first writes (sequence, own length) per row for the
// kernels and lets every length grow by one afterwards, on the device and in the host copy.
static int decode_forward(pt_handle* h, const pt_workspace& w, const int32_t* dev_tokens, const float* dev_hidden_in,
                          int32_t hidden_tracks, int32_t B, float* dev_logits, float* dev_hidden_out, int32_t* dev_argmax) {
  int rc;
  const int mode = dev_logits ? PT_LOGITS_LAST : PT_LOGITS_NONE;
  if (h->ragged) {
    int4* seq_info = (int4*)(h->kv + h->lay.off_seq);
    int2* row_map = (int2*)(w.base + w.off_rowmap);
    rc = pt_launch_decode_rowmap(seq_info, B, row_map, h->stream);
    if (rc) return rc;
    ragged_ctx rg;
    memset(&rg, 0, sizeof(rg));
    rg.row_map = row_map;
    rg.max_pos = h->seq_len;
    rc = forward(h, w, dev_tokens, dev_hidden_in, hidden_tracks, B, 1, h->seq_len, mode, dev_logits, dev_hidden_out, dev_argmax, &rg);
    h->active = &h->arena;
    if (rc) return rc;
    rc = pt_launch_advance_lens(seq_info, B, h->stream);
    if (rc) return rc;
    for (pt_seq& q : h->seqs) q.len += 1;
  } else {
    rc = forward(h, w, dev_tokens, dev_hidden_in, hidden_tracks, B, 1, h->seq_len, mode, dev_logits, dev_hidden_out, dev_argmax);
    h->active = &h->arena;
    if (rc) return rc;
  }
  h->seq_len += 1;
  return PT_OK;
}

extern "C" int pt_decode_step(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                              int32_t hidden_tracks, int32_t B, float* dev_logits,
                              float* dev_hidden_out, int32_t* dev_argmax) {
  int rc = decode_checks(h, dev_tokens, dev_hidden_in, hidden_tracks, B, dev_logits, dev_argmax);
  if (rc) return rc;
  return decode_forward(h, h->arena, dev_tokens, dev_hidden_in, hidden_tracks, B, dev_logits, dev_hidden_out, dev_argmax);
}

// ---------------------------------------------------------------------------------------------
// pt_decode_step_static: the decode step for callers that cannot allocate.  Every temporary of the step lives
// in `scratch`, a file-scope device array that each GPU holds from library load to process end.  In host code
// the array's name is only a handle for hipGetSymbolAddress; the device address obtained from it (once per
// device, with that device current) is what kernels and fills receive.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[PT_STATIC_SCRATCH_BYTES];

enum { PT_MAX_DEVICES = 64 };
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[PT_MAX_DEVICES];   // device address of `scratch` on each device, once resolved

static int static_scratch_base(char** out) {
  int dev = -1;
  PT_HIP_CHECK(hipGetDevice(&dev));
  if (dev < 0 || dev >= PT_MAX_DEVICES) return pt_set_error(PT_ERR_HIP, "device ordinal %d out of range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    PT_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return pt_set_error(PT_ERR_HIP, "hipGetSymbolAddress returned a null address for the static scratch array");
    g_scratch_ptr[dev] = (char*)p;
  }
  *out = g_scratch_ptr[dev];
  return PT_OK;
}

extern "C" int pt_decode_step_static(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                                     int32_t hidden_tracks, int32_t B, float* dev_logits,
                                     float* dev_hidden_out, int32_t* dev_argmax) {
  int rc = decode_checks(h, dev_tokens, dev_hidden_in, hidden_tracks, B, dev_logits, dev_argmax);
  if (rc) return rc;
  const pt_config& c = h->cfg;
  // Temporaries of B rows per track.  Decode attention cuts a sequence into at most ceil(1024 / (tracks *
  // sequences * KV heads)) key ranges; the K-slice area of the decode GEMMs gets what is left of the array.
  const int64_t groups = (int64_t)c.n_tracks * B * c.n_kv_heads;
  int32_t splits = (int32_t)((1024 + groups - 1) / groups);
  if (splits > PT_MAX_SPLITS) splits = PT_MAX_SPLITS;
  pt_workspace w;
  pt_layout_workspace(&c, &h->lay, B, B, 0, splits, &w);
  if (w.bytes > (size_t)PT_STATIC_SCRATCH_BYTES)
    return pt_set_error(PT_ERR_CAPACITY, "a decode step of this model at batch %d needs %zu bytes of temporaries; the "
                        "static scratch array holds %d", B, w.bytes, (int)PT_STATIC_SCRATCH_BYTES);
  w.skp_floats = (int64_t)((size_t)PT_STATIC_SCRATCH_BYTES - w.bytes) / 4;
  if (w.skp_floats > PT_SK_PART_FLOATS) w.skp_floats = PT_SK_PART_FLOATS;
  rc = static_scratch_base(&w.base);
  if (rc) return rc;
  return decode_forward(h, w, dev_tokens, dev_hidden_in, hidden_tracks, B, dev_logits, dev_hidden_out, dev_argmax);
}

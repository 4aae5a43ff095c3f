// Weight initialisation (a second, independent implementation of the repository's counter-based
// normal generator) and logical <-> physical weight copies.
//
// Generator: stream key = mix64(mix64(seed + GAMMA) ^ tag(kind, track, layer)); counter c gives
// z = mix64(key + (c + 1) * GAMMA); u1 = (hi32(z) + 1) / 2^32, u2 = lo32(z) / 2^32; Box-Muller with
// ln() and sin/cos evaluated by fixed polynomials that use only + - * / sqrt in double, one
// rounding per operation.  Fused multiply-add must therefore stay off in this file.
#pragma clang fp contract(off)

#include <string.h>

#include "pt_device.h"

#define PT_GAMMA 0x9E3779B97F4A7C15ULL

__host__ __device__ static inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}

static uint64_t stream_key(uint64_t seed, uint32_t kind, uint32_t track, uint32_t layer) {
  const uint64_t tag = ((uint64_t)(kind & 0xFFFFu) << 40) | ((uint64_t)(track & 0xFFFFFu) << 20) | (uint64_t)(layer & 0xFFFFFu);
  return mix64(mix64(seed + PT_GAMMA) ^ tag);
}

__device__ static double log_poly(double u) {
  const long long bits = __double_as_longlong(u);
  int e = (int)((bits >> 52) & 0x7ff) - 1022;
  double m = __longlong_as_double((bits & 0x800FFFFFFFFFFFFFLL) | (1022LL << 52));  // [0.5, 1)
  if (m < 0.7071067811865476) {
    m = m * 2.0;
    e -= 1;
  }
  const double s = (m - 1.0) / (m + 1.0);
  const double s2 = s * s;
  double p = 1.0 / 19.0;
  p = p * s2 + (1.0 / 17.0);
  p = p * s2 + (1.0 / 15.0);
  p = p * s2 + (1.0 / 13.0);
  p = p * s2 + (1.0 / 11.0);
  p = p * s2 + (1.0 / 9.0);
  p = p * s2 + (1.0 / 7.0);
  p = p * s2 + (1.0 / 5.0);
  p = p * s2 + (1.0 / 3.0);
  p = p * s2 + (1.0 / 1.0);
  return (2.0 * s) * p + (double)e * 0.6931471805599453;
}

__device__ static void sincos_poly(double a, double* c, double* s) {
  const double a2 = a * a;
  double sp = -1.0 / 1307674368000.0;
  sp = sp * a2 + (1.0 / 6227020800.0);
  sp = sp * a2 + (1.0 / -39916800.0);
  sp = sp * a2 + (1.0 / 362880.0);
  sp = sp * a2 + (1.0 / -5040.0);
  sp = sp * a2 + (1.0 / 120.0);
  sp = sp * a2 + (1.0 / -6.0);
  sp = sp * a2 + (1.0 / 1.0);
  *s = a * sp;
  double cp = 1.0 / 20922789888000.0;
  cp = cp * a2 + (1.0 / -87178291200.0);
  cp = cp * a2 + (1.0 / 479001600.0);
  cp = cp * a2 + (1.0 / -3628800.0);
  cp = cp * a2 + (1.0 / 40320.0);
  cp = cp * a2 + (1.0 / -720.0);
  cp = cp * a2 + (1.0 / 24.0);
  cp = cp * a2 + (1.0 / -2.0);
  cp = cp * a2 + (1.0 / 1.0);
  *c = cp;
}

// the two standard normals of counter c
__device__ static void normal_pair(uint64_t key, uint64_t c, double* n0, double* n1) {
  const uint64_t z = mix64(key + (c + 1) * PT_GAMMA);
  const double hi = (double)(uint32_t)(z >> 32), lo = (double)(uint32_t)(z & 0xFFFFFFFFu);
  const double u1 = (hi + 1.0) * (1.0 / 4294967296.0);
  const double u2 = lo * (1.0 / 4294967296.0);
  const double r = sqrt(-2.0 * log_poly(u1));
  const double t = u2 * 4.0;
  const double q = floor(t);
  const double a = ((t - q) - 0.5) * 1.5707963267948966;
  double c0, s0;
  sincos_poly(a, &c0, &s0);
  const int qi = (int)q;
  const double cc = qi == 0 ? c0 : (qi == 1 ? -s0 : (qi == 2 ? -c0 : s0));
  const double ss = qi == 0 ? s0 : (qi == 1 ? c0 : (qi == 2 ? -s0 : -c0));
  *n0 = r * cc;
  *n1 = r * ss;
}

// Where logical element (r, c) of a tensor lives: base[prow(c) * ld + r] (transposed storage with an
// optional 32-row gate/up interleave) or base[r * ld + c] (plain).
struct wmap {
  void* base;
  int64_t rows, cols, ld;
  int64_t row_off;    // added to the physical row
  int32_t interleave; // 0: none, 1: gate slot, 2: up slot of the 64-row gate/up groups
  int32_t transposed;
  int32_t dtype;      // storage type
};

__device__ static inline int64_t phys_index(const wmap& m, int64_t r, int64_t c) {
  if (!m.transposed) return r * m.ld + c;
  int64_t pr = c;
  if (m.interleave) pr = (c / 32) * 64 + (m.interleave == 2 ? 32 : 0) + (c % 32);
  return (m.row_off + pr) * m.ld + r;
}

__device__ static inline void store_w(const wmap& m, int64_t idx, float v) {
  if (m.dtype == PT_F32) ((float*)m.base)[idx] = v;
  else ((bf16_t*)m.base)[idx] = f32_to_bf16(v);
}
__device__ static inline float load_w(const wmap& m, int64_t idx) {
  return m.dtype == PT_F32 ? ((const float*)m.base)[idx] : bf16_to_f32(((const bf16_t*)m.base)[idx]);
}

// one thread per logical pair (r, 2*cp), (r, 2*cp + 1); r runs fastest so that transposed stores coalesce
__global__ void __launch_bounds__(256) init_normal_kernel(wmap m, uint64_t key, double std_dev) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t half_cols = m.cols / 2;
  if (idx >= m.rows * half_cols) return;
  int64_t r, cp;
  if (m.transposed) { r = idx % m.rows; cp = idx / m.rows; }
  else { cp = idx % half_cols; r = idx / half_cols; }
  const uint64_t counter = (uint64_t)(r * half_cols + cp);   // = (r*cols + 2*cp) >> 1
  double n0, n1;
  normal_pair(key, counter, &n0, &n1);
  store_w(m, phys_index(m, r, 2 * cp), (float)(n0 * std_dev));
  store_w(m, phys_index(m, r, 2 * cp + 1), (float)(n1 * std_dev));
}

// one thread per logical element (any column count): element e takes normal e & 1 of counter e >> 1
__global__ void __launch_bounds__(256) init_normal_elem_kernel(wmap m, uint64_t key, double std_dev) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= m.rows * m.cols) return;
  const int64_t r = idx % m.rows, c = idx / m.rows;
  const int64_t e = r * m.cols + c;
  double n0, n1;
  normal_pair(key, (uint64_t)(e >> 1), &n0, &n1);
  store_w(m, phys_index(m, r, c), (float)(((e & 1) ? n1 : n0) * std_dev));
}

__global__ void __launch_bounds__(256) weight_copy_kernel(wmap m, float* logical, int to_storage) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= m.rows * m.cols) return;
  int64_t r, c;
  if (m.transposed) { r = idx % m.rows; c = idx / m.rows; }
  else { c = idx % m.cols; r = idx / m.cols; }
  const int64_t p = phys_index(m, r, c);
  if (to_storage) store_w(m, p, logical[r * m.cols + c]);
  else logical[r * m.cols + c] = load_w(m, p);
}

static int make_map(const pt_handle* h, int32_t tensor, int32_t track, int32_t layer, wmap* m) {
  const pt_config& c = h->cfg;
  const pt_layout& l = h->lay;
  const int64_t es = l.elem_size, d = c.d_model, f = c.d_ffn;
  // PT-MoE: the feed-forward tensors exist once per expert, addressed with layer = PT_EXPERT_LAYER(layer, expert)
  int64_t expert = 0;
  if (c.n_experts > 0 && (tensor == PT_W_G || tensor == PT_W_U || tensor == PT_W_D)) {
    expert = (layer >> 12) - 1;
    layer &= 0xfff;
    if (expert < 0 || expert >= c.n_experts) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "expert %d out of range", (int)expert);
  }
  char* lw = h->w + l.off_layers + (size_t)(((int64_t)track * c.n_layers + layer) * l.layer_w_elems * es);
  char* le = lw + (l.off_exp_elems + expert * l.expert_elems) * es;   // this expert's gate/up block, then its down block
  memset(m, 0, sizeof(*m));
  m->dtype = c.dtype;
  m->transposed = 1;
  switch (tensor) {
    case PT_W_Q: m->base = lw; m->rows = d; m->cols = l.hq; m->ld = d; m->row_off = 0; break;
    case PT_W_K: m->base = lw; m->rows = d; m->cols = l.hk; m->ld = d; m->row_off = l.hq; break;
    case PT_W_V: m->base = lw; m->rows = d; m->cols = l.hk; m->ld = d; m->row_off = l.hq + l.hk; break;
    case PT_W_O: m->base = lw + l.wqkv_elems * es; m->rows = l.hq; m->cols = d; m->ld = l.hq; break;
    case PT_W_G: m->base = le; m->rows = d; m->cols = f; m->ld = d; m->interleave = 1; break;
    case PT_W_U: m->base = le; m->rows = d; m->cols = f; m->ld = d; m->interleave = 2; break;
    case PT_W_D: m->base = le + l.wgu_elems * es; m->rows = f; m->cols = d; m->ld = f; break;
    case PT_W_ROUTER: m->base = lw + l.off_wr_elems * es; m->rows = d; m->cols = c.n_experts; m->ld = d; break;
    case PT_W_EMBED: m->base = h->w + l.off_embed; m->rows = c.vocab; m->cols = d; m->ld = d; m->transposed = 0; break;
    case PT_W_HEAD: m->base = h->w + l.off_headT; m->rows = d; m->cols = c.vocab; m->ld = d; break;
    case PT_W_G1:
    case PT_W_G2:
      m->base = h->w + l.off_gains + (size_t)((((int64_t)track * c.n_layers + layer) * 2 + (tensor == PT_W_G2)) * d * 4);
      m->rows = 1; m->cols = d; m->ld = d; m->transposed = 0; m->dtype = PT_F32; break;
    case PT_W_GF: m->base = h->w + l.off_gf; m->rows = 1; m->cols = d; m->ld = d; m->transposed = 0; m->dtype = PT_F32; break;
    default: return pt_set_error(PT_ERR_INVALID_ARGUMENT, "unknown tensor id %d", tensor);
  }
  return PT_OK;
}

int pt_launch_weight_copy(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, float* logical, bool to_storage) {
  wmap m;
  int rc = make_map(h, tensor, track, layer, &m);
  if (rc) return rc;
  const int64_t n = m.rows * m.cols;
  hipLaunchKernelGGL(weight_copy_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, h->stream, m, logical, to_storage ? 1 : 0);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

int pt_launch_weight_init(pt_handle* h, uint64_t seed) {
  const pt_config& c = h->cfg;
  const pt_layout& l = h->lay;
  const double sd = (double)c.init_std;
  static const int32_t per_layer[7] = {PT_W_Q, PT_W_K, PT_W_V, PT_W_O, PT_W_G, PT_W_U, PT_W_D};
  wmap m;
  for (int t = 0; t < c.n_tracks; ++t)
    for (int layer = 0; layer < c.n_layers; ++layer) {
      for (int k = 0; k < 7; ++k) {
        const bool per_expert = c.n_experts > 0 && k >= 4;
        for (int e = 0; e < (per_expert ? c.n_experts : 1); ++e) {
          const int32_t lay = per_expert ? PT_EXPERT_LAYER(layer, e) : layer;   // also the stream's layer field
          int rc = make_map(h, per_layer[k], t, lay, &m);
          if (rc) return rc;
          const int64_t n = m.rows * (m.cols / 2);
          hipLaunchKernelGGL(init_normal_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, h->stream, m,
                             stream_key(seed, (uint32_t)per_layer[k], (uint32_t)t, (uint32_t)lay), sd);
        }
      }
      if (c.n_experts > 0) {
        int rc = make_map(h, PT_W_ROUTER, t, layer, &m);
        if (rc) return rc;
        const int64_t n = m.rows * m.cols;
        hipLaunchKernelGGL(init_normal_elem_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, h->stream, m,
                           stream_key(seed, PT_W_ROUTER, (uint32_t)t, (uint32_t)layer), sd);
      }
    }
  if (c.vocab > 0) {
    for (int32_t tensor : {PT_W_EMBED, PT_W_HEAD}) {
      int rc = make_map(h, tensor, 0, 0, &m);
      if (rc) return rc;
      const int64_t n = m.rows * (m.cols / 2);
      hipLaunchKernelGGL(init_normal_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, h->stream, m,
                         stream_key(seed, (uint32_t)tensor, 0, 0), sd);
    }
  }
  PT_HIP_CHECK(hipGetLastError());
  int rc = pt_launch_fill_f32((float*)(h->w + l.off_gains), (int64_t)c.n_tracks * c.n_layers * 2 * c.d_model, 1.0f, h->stream);
  if (rc) return rc;
  return pt_launch_fill_f32((float*)(h->w + l.off_gf), c.d_model, 1.0f, h->stream);
}

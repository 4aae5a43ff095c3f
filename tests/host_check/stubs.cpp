// Host-only build of the library's call sequencing (csrc/pt_api.cpp) for the sanitizer test: every kernel
// launcher is replaced by a function that launches nothing and instead checks that each buffer the real kernel
// would touch lies inside memory the caller registered (the three arenas, the static scratch array, the caller's
// input and output buffers).  The HIP runtime calls pt_api.cpp makes are replaced as well, so the program runs
// without a GPU.  A violation prints what overflowed and aborts.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "pt_internal.h"
#include "host_check.h"

namespace {
struct range { uintptr_t lo, hi; const char* name; };
std::vector<range> g_ranges;
long g_checked = 0, g_launches = 0;
int g_mode = 0;

void need(const void* p, double bytes, const char* what) {
  if (bytes <= 0) return;
  ++g_checked;
  const uintptr_t lo = (uintptr_t)p, hi = lo + (uintptr_t)bytes;
  for (const range& r : g_ranges)
    if (lo >= r.lo && hi <= r.hi) return;
  fprintf(stderr, "host_check: %s = [%#zx, %#zx) (%.0f bytes) lies in no registered buffer\n", what, (size_t)lo, (size_t)hi, bytes);
  for (const range& r : g_ranges) fprintf(stderr, "  %-10s [%#zx, %#zx)\n", r.name, (size_t)r.lo, (size_t)r.hi);
  abort();
}
int esize(int dtype) { return dtype == PT_F32 ? 4 : 2; }

// operands of a GEMM, from the fields the kernels read
void check_gemm(const pt_gemm_args& g, const char* who) {
  ++g_launches;
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return;
  const int es = esize(g.dtype);
  const int groups = g.blk_group ? (g.n_groups > 0 ? g.n_groups : 1) : 1;
  for (int b = 0; b < g.batch; ++b) {
    if (g.norm_src) {
      need(g.norm_src + b * g.norm_bstride, ((double)(g.M - 1) * g.K + g.K) * 4, "GEMM norm_src");
      need(g.norm_gain + b * g.norm_gbstride, g.K * 4.0, "GEMM norm_gain");
    } else if (g.a_rows) {
      // gathered rows: any row of the track's A may be read; the table itself holds M entries
      need(g.a_rows + b * g.a_rows_bstride, g.M * 4.0, "GEMM a_rows");
      if (g.a_bstride <= 0 || g.a_bstride % g.lda) { fprintf(stderr, "host_check: %s gathers rows but a_bstride is not a whole number of rows\n", who); abort(); }
      need((const char*)g.A + (size_t)b * g.a_bstride * es, (double)g.a_bstride * es, "GEMM A (gathered)");
    } else {
      need((const char*)g.A + (size_t)b * g.a_bstride * es, ((double)(g.M - 1) * g.lda + g.K) * es, "GEMM A");
    }
    for (int e = 0; e < groups; ++e)
      need((const char*)g.W + ((size_t)b * g.w_bstride + (size_t)e * g.w_gstride) * es, ((double)(g.N - 1) * g.ldb + g.K) * es, "GEMM W");
    if (g.blk_group) need(g.blk_group + b * g.grp_bstride, (g.M / 64) * 4.0, "GEMM blk_group");
    if (g.grp_count) {
      need(g.grp_count + b * g.grp_info_bstride, g.n_groups * 4.0, "GEMM grp_count");
      need(g.grp_base + b * g.grp_info_bstride, g.n_groups * 4.0, "GEMM grp_base");
    }
    if (g.rs_inv) need(g.rs_inv + b * g.rs_bstride, g.M * 4.0, "GEMM rs_inv");
    if (g.epi == EPI_STORE_F32 || g.epi == EPI_RESIDUAL) {
      need(g.out + b * g.out_bstride, ((double)(g.M - 1) * g.ldo + g.N) * 4, "GEMM out");
      if (g.epi == EPI_RESIDUAL) need(g.res + b * g.res_bstride, ((double)(g.M - 1) * g.ldo + g.N) * 4, "GEMM res");
      if (g.nf_out) {
        need((const char*)g.nf_out + (size_t)b * g.nf_out_bstride * 2, (double)g.M * g.N * 2, "GEMM nf_out");
        need(g.nf_gain + b * g.nf_gain_bstride, g.N * 4.0, "GEMM nf_gain");
        need(g.nf_ss + b * g.nf_ss_bstride, (double)g.M * g.nf_parts * 4, "GEMM nf_ss");
      }
    } else if (g.epi == EPI_SWIGLU) {
      need((const char*)g.olp + (size_t)b * g.olp_bstride * es, (double)g.M * (g.N / 2) * es, "GEMM SwiGLU out");
    } else {
      need((const char*)g.olp + (size_t)b * g.olp_bstride * es, (double)g.M * g.H * g.hd * es, "GEMM q out");
      need(g.rope, (double)(g.row_map ? 1 : g.pos0 + g.S) * g.hd * 4, "GEMM rope table");
      if (g.row_map) need(g.row_map, g.M * 8.0, "GEMM row_map");
      // last cache head this track can touch: sequences 0 .. nseq-1, kv heads 0 .. Hkv-1
      const int64_t nseq = g.row_map ? 1 : (g.M + g.S - 1) / g.S;
      const int64_t last_head = b * g.kv_bstride + (nseq - 1) * g.kv_seq_stride + g.Hkv - 1;
      need((const char*)g.kc + (size_t)b * g.kv_bstride * g.kv_head_elems * es, 1, "GEMM K cache (first head)");
      need((const char*)g.kc + (size_t)last_head * g.kv_head_elems * es, (double)g.kv_head_elems * es, "GEMM K cache (last head)");
      need((const char*)g.vc + (size_t)last_head * g.hd * g.s_pad * es, (double)g.hd * g.s_pad * es, "GEMM V cache (last head)");
    }
  }
}

void check_attn(const pt_attn_args& a) {
  ++g_launches;
  const int es = esize(a.dtype);
  const int64_t rows = a.seq_info ? a.rows : (int64_t)a.B * a.S;
  for (int t = 0; t < a.n_tracks; ++t) {
    need((const char*)a.q + (size_t)t * a.q_bstride * es, (double)rows * a.H * a.hd * es, "attention q");
    need((const char*)a.o + (size_t)t * a.q_bstride * es, (double)rows * a.H * a.hd * es, "attention o");
    const int64_t last_head = t * a.kv_bstride + (int64_t)(a.B - 1) * a.kv_seq_stride + a.Hkv - 1;
    need((const char*)a.kc + (size_t)last_head * a.kv_head_elems * es, (double)a.kv_head_elems * es, "attention K cache");
    need((const char*)a.vc + (size_t)last_head * a.hd * a.s_pad * es, (double)a.hd * a.s_pad * es, "attention V cache");
  }
  if (a.S == 1 && a.partials)
    need(a.partials, (double)a.n_tracks * a.B * a.H * a.max_splits * (a.hd + 2) * 4, "attention split partials");
  if (a.row_map) need(a.row_map, (a.S == 1 ? a.B : rows) * 8.0, "attention row_map");
  if (a.seq_info) need(a.seq_info, a.B * 16.0, "attention seq_info");
  const int64_t max_key = a.row_map ? (a.S == 1 ? a.max_pos : a.max_plen - 1) : (int64_t)a.pos0 + a.S - 1;
  if (max_key >= a.kv_head_elems / a.hd || max_key >= a.s_pad) {
    fprintf(stderr, "host_check: attention reads key %lld past the cache rows\n", (long long)max_key);
    abort();
  }
}
}  // namespace

extern "C" void hc_add_range(const void* p, size_t bytes, const char* name) { g_ranges.push_back({(uintptr_t)p, (uintptr_t)p + bytes, name}); }
extern "C" void hc_clear_ranges(void) { g_ranges.clear(); }
extern "C" void hc_set_mode(int mode) { g_mode = mode; }
extern "C" long hc_checked(void) { return g_checked; }
extern "C" long hc_launches(void) { return g_launches; }

// ------------------------------------------------------------------------------------------------ GEMM family
// mode 0: the tuned kernels refuse everything (generic path); mode 1: they take everything they are offered,
// fold the norm where asked and split K in the decode residual GEMMs.
int pt_tune_gemm_cfg = -1, pt_tune_skinny_plan = 0, pt_tune_attn_prefill = 0;
int pt_launch_gemm_generic(const pt_gemm_args& g, hipStream_t) { check_gemm(g, "generic GEMM"); return PT_OK; }
bool pt_gemm_mfma_covers(const pt_gemm_args& g) { return g_mode == 1 && g.dtype == PT_BF16 && g.K % 128 == 0; }
int pt_launch_gemm_mfma(const pt_gemm_args& g, hipStream_t) {
  if (!pt_gemm_mfma_covers(g)) return 0;
  check_gemm(g, "MFMA GEMM");
  return 1;
}
int pt_gemm_mfma_fold_parts(const pt_gemm_args& g) {
  return pt_gemm_mfma_covers(g) && g.epi == EPI_RESIDUAL && g.N % 128 == 0 ? g.N / 128 : 0;
}
static bool skinny_ok(const pt_gemm_args& g) { return g_mode == 1 && g.dtype == PT_BF16 && g.K % 512 == 0 && g.N % 32 == 0; }
int pt_gemm_skinny_ksplit(const pt_gemm_args& g) {
  if (!skinny_ok(g) || g.M > 64) return 0;
  if (g.epi != EPI_RESIDUAL || !g.sk_part) return 1;
  int ks = 4;
  while (ks > 1 && ((int64_t)ks * g.batch * g.M * g.N > g.sk_part_floats || g.K % (ks * 512))) --ks;
  return ks;
}
bool pt_gemm_fuses_norm(const pt_gemm_args& g) { return skinny_ok(g) && g.M <= 4 && (g.epi == EPI_QKV || g.epi == EPI_SWIGLU) && g.lda == g.K; }
int pt_launch_gemm_skinny(const pt_gemm_args& g_in, bool allow_split, hipStream_t) {
  pt_gemm_args g = g_in;
  if (g.n_groups > 0) {
    if (g.grp_max_rows > 64) return 0;
    g.M = g.grp_max_rows;   // rows of one group; outputs are checked over the whole slot range below
  }
  if (!skinny_ok(g) || g.M > 64) return 0;
  if (g.norm_src && !pt_gemm_fuses_norm(g)) return 0;
  check_gemm(g_in, "weight-streaming GEMM");
  if (allow_split && pt_gemm_skinny_ksplit(g) > 1)
    need(g.sk_part, (double)pt_gemm_skinny_ksplit(g) * g.batch * g.M * g.N * 4, "GEMM K slices");
  return g.M <= 4 && g.n_groups == 0 ? 3 : 2;
}

// ------------------------------------------------------------------------------------------------ attention
int pt_launch_attn_generic(const pt_attn_args& a, hipStream_t) { check_attn(a); return PT_OK; }
int pt_launch_attn_prefill_mfma(const pt_attn_args& a, hipStream_t) {
  if (g_mode == 0 || a.dtype != PT_BF16 || (a.hd != 64 && a.hd != 128) || a.S % 32) return 0;
  check_attn(a);
  return 1;
}
int pt_launch_attn_decode(const pt_attn_args& a, hipStream_t) {
  if (g_mode == 0 || a.dtype != PT_BF16 || (a.hd != 64 && a.hd != 128)) return 0;
  check_attn(a);
  return 1;
}

// ------------------------------------------------------------------------------------------------ the rest
int pt_launch_embed(const void* embed, int32_t dtype, const int32_t* tokens, int64_t rows, int32_t d, int32_t vocab,
                    float* h, int32_t* flag, hipStream_t) {
  ++g_launches;
  need(embed, (double)vocab * d * esize(dtype), "embedding table");
  need(tokens, rows * 4.0, "tokens");
  need(h, (double)rows * d * 4, "embedding out");
  need(flag, 4, "status word");
  return PT_OK;
}
int pt_launch_embed_ragged(const void* embed, int32_t dtype, const int32_t* tokens, const int2* row_map, const int4* seq_info,
                           int64_t rows, int32_t d, int32_t vocab, float* h, int32_t* flag, hipStream_t) {
  ++g_launches;
  need(embed, (double)vocab * d * esize(dtype), "embedding table");
  need(tokens, 4, "tokens");
  need(row_map, rows * 8.0, "row_map");
  need(seq_info, 16, "seq_info");
  need(h, (double)rows * d * 4, "embedding out");
  need(flag, 4, "status word");
  return PT_OK;
}
int pt_launch_scatter_rows(const float* src, int64_t src_bstride, const int2* row_map, const int4* seq_info, int64_t rows,
                           int32_t d, int32_t batch, float* dst, int64_t dst_bstride, hipStream_t) {
  ++g_launches;
  need(src + (batch - 1) * src_bstride, 4, "scatter src");
  need(row_map, rows * 8.0, "row_map");
  need(seq_info, 16, "seq_info");
  need(dst + (batch - 1) * dst_bstride, (double)rows * d * 4, "scatter dst");
  return PT_OK;
}
int pt_launch_gather_rows(const float* src, const int32_t* idx, int64_t n, int32_t d, float* dst, hipStream_t) {
  ++g_launches;
  need(src, 4, "gather src");
  need(idx, n * 4.0, "gather index");
  need(dst, (double)n * d * 4, "gather dst");
  return PT_OK;
}
int pt_launch_ragged_maps(const int4* seq_info, int32_t B, int64_t rows, int2* row_map, int32_t* valid, int32_t* last, hipStream_t) {
  ++g_launches;
  need(seq_info, B * 16.0, "seq_info");
  need(row_map, rows * 8.0, "row_map");
  need(valid, rows * 4.0, "valid rows");   // at most one entry per packed row
  need(last, B * 4.0, "last rows");
  return PT_OK;
}
int pt_launch_decode_rowmap(int4* seq_info, int32_t B, int2* row_map, hipStream_t) {
  ++g_launches;
  need(seq_info, B * 16.0, "seq_info");
  need(row_map, B * 8.0, "row_map");
  return PT_OK;
}
int pt_launch_advance_lens(int4* seq_info, int32_t B, hipStream_t) { ++g_launches; need(seq_info, B * 16.0, "seq_info"); return PT_OK; }
int pt_launch_rmsnorm(const float* h, int64_t h_bstride, const float* gains, int64_t g_bstride, void* out, int64_t out_bstride,
                      int32_t dtype, int32_t batch, int64_t rows, int32_t d, float, hipStream_t) {
  ++g_launches;
  for (int b = 0; b < batch; ++b) {
    need(h + b * h_bstride, (double)rows * d * 4, "rmsnorm in");
    need(gains + b * g_bstride, d * 4.0, "rmsnorm gain");
    need((char*)out + (size_t)b * out_bstride * esize(dtype), (double)rows * d * esize(dtype), "rmsnorm out");
  }
  return PT_OK;
}
int pt_launch_rmsnorm_rows(const float* h, const float* gain, void* out, int32_t dtype, int64_t rows, int64_t row_step,
                           int64_t row_off, const int32_t* row_idx, int32_t d, float, hipStream_t) {
  ++g_launches;
  if (row_idx) need(row_idx, rows * 4.0, "rmsnorm row index");
  else need(h + ((rows - 1) * row_step + row_off) * d, d * 4.0, "rmsnorm last input row");
  need(gain, d * 4.0, "rmsnorm gain");
  need(out, (double)rows * d * esize(dtype), "rmsnorm out");
  return PT_OK;
}
int pt_launch_merge(const void* const* tracks, int32_t n, int64_t elems, int32_t dtype, float, void* out, float* tap, hipStream_t) {
  ++g_launches;
  for (int i = 0; i < n; ++i) need(tracks[i], (double)elems * esize(dtype), "merge input");
  need(out, (double)elems * esize(dtype), "merge out");
  if (tap) need(tap, elems * 4.0, "merge tap");
  return PT_OK;
}
int pt_launch_copy_f32(const float* src, float* dst, int64_t elems, hipStream_t) {
  ++g_launches;
  need(src, elems * 4.0, "copy src");
  need(dst, elems * 4.0, "copy dst");
  return PT_OK;
}
int pt_launch_argmax(const float* logits, int32_t rows, int32_t vocab, int32_t* out, hipStream_t) {
  ++g_launches;
  need(logits, (double)rows * vocab * 4, "argmax logits");
  need(out, rows * 4.0, "argmax out");
  return PT_OK;
}
int pt_launch_rope_table(float* table, int32_t max_seq, int32_t hd, float, hipStream_t) { ++g_launches; need(table, (double)max_seq * hd * 4, "rope table"); return PT_OK; }
int pt_launch_resnorm(const float* part, int32_t slices, const float* res, int64_t res_bstride, float* h, int64_t h_bstride,
                      const float* gains, int64_t g_bstride, void* out, int64_t out_bstride, int32_t batch, int64_t rows, int32_t d,
                      float, hipStream_t) {
  ++g_launches;
  need(part, (double)slices * batch * rows * d * 4, "K slices");
  for (int b = 0; b < batch; ++b) {
    need(res + b * res_bstride, (double)rows * d * 4, "resnorm residual");
    need(h + b * h_bstride, (double)rows * d * 4, "resnorm stream");
    if (out) {
      need(gains + b * g_bstride, d * 4.0, "resnorm gain");
      need((char*)out + (size_t)b * out_bstride * 2, (double)rows * d * 2, "resnorm out");
    }
  }
  return PT_OK;
}
int pt_launch_fill_f32(float* dst, int64_t n, float, hipStream_t) { ++g_launches; need(dst, n * 4.0, "fill"); return PT_OK; }
int pt_launch_row_inv_rms(const float* ss, int32_t parts, int64_t rows, int32_t, float, float* out, hipStream_t) {
  ++g_launches;
  need(ss, (double)rows * parts * 4, "row sums of squares");
  need(out, rows * 4.0, "row factors");
  return PT_OK;
}
int pt_launch_moe_route(const pt_moe_args& a, hipStream_t) {
  ++g_launches;
  const double n = (double)a.T * a.rows;
  const int64_t nblk = (a.rows + 255) / 256;
  need(a.logits, n * a.e_pad * 4, "router logits");
  need(a.route, n * a.k * 4, "chosen experts");
  need(a.gate, n * a.k * 4, "gates");
  need(a.slot, n * a.k * 4, "slots");
  need(a.perm, (double)a.T * a.slots * 4, "row of slot");
  need(a.blk, (double)a.T * (a.slots / 64) * 4, "expert of block");
  need(a.cnt, (double)a.T * (nblk + 2) * 64 * 4, "expert counts");
  need(a.flag, 4, "status word");
  for (int t = 0; t < a.T; ++t) {
    if (a.forced) need(a.forced + t * a.obs_bstride, (double)a.rows * a.k * 4, "prescribed experts");
    if (a.chosen_out) need(a.chosen_out + t * a.obs_bstride, (double)a.rows * a.k * 4, "observed experts");
  }
  if (a.slots < a.rows * a.k + (int64_t)a.E * 255 || a.slots % 256) { fprintf(stderr, "host_check: too few expert slots\n"); abort(); }
  return PT_OK;
}
int pt_launch_moe_combine(const pt_moe_args& a, const float* y, const float* res, int64_t res_bstride, float* h, int32_t d,
                          const float* gains, int64_t g_bstride, void* out, int32_t dtype, float, hipStream_t) {
  ++g_launches;
  need(y, (double)a.T * a.slots * d * 4, "expert outputs");
  need(h, (double)a.T * a.rows * d * 4, "combine stream");
  for (int t = 0; t < a.T; ++t) {
    need(res + t * res_bstride, (double)a.rows * d * 4, "combine residual");
    if (out) need(gains + t * g_bstride, d * 4.0, "combine gain");
  }
  if (out) need(out, (double)a.T * a.rows * d * esize(dtype), "combine normed out");
  return PT_OK;
}
int pt_launch_weight_init(pt_handle* h, uint64_t) { ++g_launches; need(h->w, (double)h->lay.weight_bytes, "weight arena"); return PT_OK; }
int pt_launch_weight_copy(pt_handle*, int32_t, int32_t, int32_t, float* logical, bool) { ++g_launches; need(logical, 4, "weight staging"); return PT_OK; }

// ------------------------------------------------------------------------------------------------ HIP runtime
// Only what pt_api.cpp calls.  Copies move nothing (the "device" memory is an address range, not storage).
static unsigned char g_fake_scratch_tag;
extern "C" {
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t bytes, hipMemcpyKind kind, hipStream_t) {
  if (kind == hipMemcpyHostToDevice) need(dst, (double)bytes, "host-to-device copy target");
  else if (kind == hipMemcpyDeviceToHost) { need(src, (double)bytes, "device-to-host copy source"); memset(dst, 0, bytes); }
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
hipError_t hipGetDevice(int* dev) { *dev = 0; return hipSuccess; }
hipError_t hipGetSymbolAddress(void** p, const void*) { *p = hc_scratch_address(); (void)g_fake_scratch_tag; return hipSuccess; }
hipError_t hipEventCreate(hipEvent_t* e) { *e = (hipEvent_t)malloc(8); return hipSuccess; }
hipError_t hipEventDestroy(hipEvent_t e) { free((void*)e); return hipSuccess; }
hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
hipError_t hipEventElapsedTime(float* ms, hipEvent_t, hipEvent_t) { *ms = 1.0f; return hipSuccess; }
const char* hipGetErrorString(hipError_t) { return "stub"; }
}

// Drives the C ABI of libpt through its whole host-side logic without a GPU: configuration checks, arena layout,
// the launch sequence of prefill / decode / ragged batches / PT-MoE, error paths.  Built with AddressSanitizer and
// UndefinedBehaviorSanitizer on the host code; the launchers are the checking stand-ins of stubs.cpp, "device memory"
// is a set of address ranges that are never dereferenced.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "pt.h"
#include "host_check.h"

#ifndef HC_SHRINK
#define HC_SHRINK 0
#endif

#define EXPECT(cond)                                                                      \
  do {                                                                                    \
    if (!(cond)) {                                                                        \
      fprintf(stderr, "driver: %s:%d: %s failed (last error: %s)\n", __FILE__, __LINE__, #cond, pt_last_error()); \
      exit(1);                                                                            \
    }                                                                                     \
  } while (0)

static char* const W_BASE = (char*)0x100000000000ull;
static char* const KV_BASE = (char*)0x200000000000ull;
static char* const WS_BASE = (char*)0x300000000000ull;
static char* const IO_BASE = (char*)0x400000000000ull;
static char* const SCRATCH_BASE = (char*)0x500000000000ull;
extern "C" void* hc_scratch_address(void) { return SCRATCH_BASE; }

// hands out caller-side "device" buffers of exact size, each its own registered range with a gap behind it
struct io_alloc {
  char* next = IO_BASE;
  void* get(size_t bytes, const char* name) {
    char* p = next;
    hc_add_range(p, bytes, name);
    next += (bytes + 4096 + 255) / 256 * 256;
    return p;
  }
};

static pt_config make(int T, int L, int D, int d, int H, int Hkv, int hd, int f, int V, int maxB, int maxS, int dtype,
                      int E = 0, int k = 0) {
  pt_config c;
  memset(&c, 0, sizeof(c));
  c.n_tracks = T; c.n_layers = L; c.block_depth = D; c.d_model = d; c.n_heads = H; c.n_kv_heads = Hkv; c.head_dim = hd;
  c.d_ffn = f; c.vocab = V; c.max_batch = maxB; c.max_seq = maxS; c.dtype = dtype;
  c.merge_scale = 1.0f / T; c.rms_eps = 1e-5f; c.rope_theta = 10000.f; c.init_std = 0.02f;
  c.n_experts = E; c.top_k = k;
  return c;
}

static void invalid_configs() {
  size_t a, b, c;
  pt_config good = make(2, 4, 2, 128, 4, 4, 32, 512, 512, 1, 64, PT_F32);
  EXPECT(pt_query_bytes(&good, &a, &b, &c) == PT_OK && a > 0 && b > 0 && c > 0);
  EXPECT(pt_query_bytes(&good, nullptr, nullptr, nullptr) == PT_OK);
  EXPECT(pt_query_bytes(nullptr, &a, &b, &c) == PT_ERR_NULL_POINTER);
  pt_config x;
  x = good; x.n_tracks = 0; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_tracks = 17; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.block_depth = 3; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.d_model = 130; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_kv_heads = 3; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.head_dim = 260; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.d_ffn = 48; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.vocab = 7; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.max_batch = 1 << 20; x.max_seq = 1 << 20; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.dtype = 5; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.rms_eps = -1.f; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_experts = 65; x.top_k = 2; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_experts = 4; x.top_k = 5; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_experts = 0; x.top_k = 1; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  x = good; x.n_experts = 16; x.top_k = 9; EXPECT(pt_query_bytes(&x, &a, &b, &c) == PT_ERR_INVALID_CONFIG);
  pt_handle* h = nullptr;
  EXPECT(pt_create(&good, W_BASE, a, KV_BASE, b, WS_BASE, c, nullptr, nullptr) == PT_ERR_NULL_POINTER);
  EXPECT(pt_create(&good, nullptr, a, KV_BASE, b, WS_BASE, c, nullptr, &h) == PT_ERR_NULL_POINTER && h == nullptr);
  EXPECT(pt_create(&good, W_BASE + 16, a, KV_BASE, b, WS_BASE, c, nullptr, &h) == PT_ERR_INVALID_ARGUMENT);
  EXPECT(pt_create(&good, W_BASE, a - 1, KV_BASE, b, WS_BASE, c, nullptr, &h) == PT_ERR_ARENA_TOO_SMALL);
  EXPECT(pt_create(&good, W_BASE, a, KV_BASE, b - 1, WS_BASE, c, nullptr, &h) == PT_ERR_ARENA_TOO_SMALL);
  EXPECT(pt_create(&good, W_BASE, a, KV_BASE, b, WS_BASE, c - 1, nullptr, &h) == PT_ERR_ARENA_TOO_SMALL);
  EXPECT(pt_destroy(nullptr) == PT_ERR_NULL_POINTER);
  EXPECT(pt_seq_len(nullptr) < 0 && pt_merge_count(nullptr) < 0);
  EXPECT(pt_set_tuning(99, 0) == PT_ERR_INVALID_ARGUMENT && pt_set_tuning(PT_TUNE_FOLD_RMSNORM, 1) == PT_OK);
}

static void run_model(const pt_config& c, int mode) {
  hc_clear_ranges();
  hc_set_mode(mode);
  size_t wb, kb, sb;
  EXPECT(pt_query_bytes(&c, &wb, &kb, &sb) == PT_OK);
  // HC_SHRINK != 0 plants an overflow (the self-test of the checker): the arenas then end before their last objects
  hc_add_range(W_BASE, wb - HC_SHRINK, "weights");
  hc_add_range(KV_BASE, kb - HC_SHRINK, "kv cache");
  hc_add_range(WS_BASE, sb, "workspace");
  hc_add_range(SCRATCH_BASE, 32u << 20, "scratch");
  io_alloc io;
  pt_handle* h = nullptr;
  EXPECT(pt_create(&c, W_BASE, wb, KV_BASE, kb, WS_BASE, sb, nullptr, &h) == PT_OK && h);
  const int T = c.n_tracks, d = c.d_model, V = c.vocab, B = c.max_batch, L = c.n_layers;
  const int S = c.max_seq >= 128 ? 96 : (c.max_seq - 8) / 32 * 32;   // leaves room for the decode steps
  const int64_t rows = (int64_t)B * S;
  int32_t* tokens = (int32_t*)io.get(rows * 4, "tokens");
  float* hidden_in = (float*)io.get((size_t)T * rows * d * 4, "hidden in");
  float* logits = V ? (float*)io.get((size_t)rows * V * 4, "logits") : nullptr;
  float* hidden_out = (float*)io.get((size_t)rows * d * 4, "hidden out");
  int32_t* amax = (int32_t*)io.get(B * 4, "argmax");
  const int merges = L / c.block_depth;
  float* taps = (float*)io.get((size_t)merges * rows * d * 4, "taps");
  float* ttaps = (float*)io.get((size_t)merges * T * rows * d * 4, "track taps");
  float* staging = (float*)io.get((size_t)4 << 20, "weight staging");

  // forward before weights exist
  EXPECT(pt_prefill(h, V ? tokens : nullptr, V ? nullptr : hidden_in, 1, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_BAD_STATE);
  EXPECT(pt_init_weights(h, 7) == PT_OK);
  EXPECT(pt_set_weight(h, PT_W_Q, 0, 0, staging) == PT_OK && pt_get_weight(h, PT_W_D, T - 1, c.n_experts ? PT_EXPERT_LAYER(L - 1, c.n_experts - 1) : L - 1, staging) == PT_OK);
  EXPECT(pt_set_weight(h, 99, 0, 0, staging) == PT_ERR_INVALID_ARGUMENT && pt_set_weight(h, PT_W_Q, T, 0, staging) == PT_ERR_INVALID_ARGUMENT);
  if (c.n_experts) {
    EXPECT(pt_get_weight(h, PT_W_ROUTER, 0, 0, staging) == PT_OK);
    EXPECT(pt_get_weight(h, PT_W_G, 0, 0, staging) == PT_ERR_INVALID_ARGUMENT);   // expert not named
    EXPECT(pt_get_weight(h, PT_W_G, 0, PT_EXPERT_LAYER(0, c.n_experts), staging) == PT_ERR_INVALID_ARGUMENT);
  } else {
    EXPECT(pt_get_weight(h, PT_W_ROUTER, 0, 0, staging) == PT_ERR_INVALID_ARGUMENT);
    EXPECT(pt_set_moe_routes(h, nullptr, nullptr) == PT_ERR_BAD_STATE);
  }
  // argument errors
  EXPECT(pt_decode_step(h, tokens, hidden_in, 1, B, logits, nullptr, nullptr) == PT_ERR_BAD_STATE);   // before prefill
  EXPECT(pt_prefill(h, tokens, hidden_in, 1, B + 1, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_CAPACITY);
  EXPECT(pt_prefill(h, tokens, hidden_in, 1, B, c.max_seq + 1, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_CAPACITY);
  EXPECT(pt_prefill(h, tokens, hidden_in, 1, 0, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);
  EXPECT(pt_prefill(h, tokens, hidden_in, 1, B, S, 7, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);
  EXPECT(pt_prefill(h, nullptr, nullptr, 1, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_NULL_POINTER);
  if (T > 2) EXPECT(pt_prefill(h, nullptr, hidden_in, 2, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);
  if (V) EXPECT(pt_prefill(h, tokens, nullptr, 1, B, S, PT_LOGITS_ALL, nullptr, nullptr) == PT_ERR_NULL_POINTER);
  else EXPECT(pt_prefill(h, tokens, nullptr, 1, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);

  EXPECT(pt_profile_enable(h, 0xffffffffu) == PT_OK);
  EXPECT(pt_set_taps(h, taps, ttaps) == PT_OK);
  int32_t* routes_out = nullptr;
  if (c.n_experts) {
    routes_out = (int32_t*)io.get((size_t)L * T * rows * c.top_k * 4, "routes out");
    int32_t* routes_in = (int32_t*)io.get((size_t)L * T * rows * c.top_k * 4, "routes in");
    EXPECT(pt_set_moe_routes(h, routes_out, routes_in) == PT_OK);
  }
  // prefill: tokens (all logits), hidden states shared and per track, last logits; other lengths
  if (V) EXPECT(pt_prefill(h, tokens, nullptr, 1, B, S, PT_LOGITS_ALL, logits, hidden_out) == PT_OK);
  EXPECT(pt_prefill(h, nullptr, hidden_in, 1, B, S, V ? PT_LOGITS_LAST : PT_LOGITS_NONE, logits, hidden_out) == PT_OK);
  EXPECT(pt_prefill(h, nullptr, hidden_in, T, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_OK);
  EXPECT(pt_merge_count(h) >= merges && pt_seq_len(h) == S);
  EXPECT(pt_set_taps(h, nullptr, nullptr) == PT_OK);
  for (int s : {1, 7, 33, 64}) {
    if (s > c.max_seq - 4) continue;
    EXPECT(pt_prefill(h, V ? tokens : nullptr, V ? nullptr : hidden_in, 1, 1, s, PT_LOGITS_NONE, nullptr, nullptr) == PT_OK);
  }
  EXPECT(pt_prefill(h, V ? tokens : nullptr, V ? nullptr : hidden_in, 1, B, S, PT_LOGITS_NONE, nullptr, nullptr) == PT_OK);
  double ms; int64_t n, fam[PT_FAMILY_COUNT];
  EXPECT(pt_profile_read(h, PT_K_GEMM_QKV, &ms, &n) == PT_OK && n > 0);
  EXPECT(pt_profile_paths(h, PT_K_GEMM_QKV, fam) == PT_OK && fam[0] + fam[1] + fam[2] + fam[3] > 0);
  EXPECT(pt_profile_read(h, 99, &ms, &n) == PT_ERR_INVALID_ARGUMENT);
  EXPECT(pt_profile_reset(h) == PT_OK && pt_profile_enable(h, 0) == PT_OK);
  // decode until the cache is full
  EXPECT(pt_decode_step(h, tokens, hidden_in, 1, B == 1 ? 2 : B - 1, logits, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);
  if (V) EXPECT(pt_decode_step(h, tokens, nullptr, 1, B, nullptr, nullptr, amax) != PT_OK);   // argmax needs logits
  int steps = 0, rc = PT_OK;
  while (true) {
    if (V && steps % 3 == 0) rc = pt_decode_step(h, tokens, nullptr, 1, B, logits, hidden_out, amax);
    else if (steps % 3 == 1) rc = pt_decode_step(h, nullptr, hidden_in, T, B, V ? logits : nullptr, hidden_out, nullptr);
    else rc = pt_decode_step(h, nullptr, hidden_in, 1, B, nullptr, hidden_out, nullptr);
    if (rc != PT_OK) break;
    ++steps;
    if (steps == 2) {   // the variant with the static scratch array: fits small batches only
      const int r2 = pt_decode_step_static(h, nullptr, hidden_in, 1, B, nullptr, hidden_out, nullptr);
      EXPECT(r2 == PT_OK || r2 == PT_ERR_CAPACITY);
      if (r2 == PT_OK) ++steps;
    }
  }
  EXPECT(rc == PT_ERR_CAPACITY && pt_seq_len(h) == c.max_seq && steps == c.max_seq - S);
  EXPECT(pt_sync_status(h) == PT_OK);
  if (c.n_experts) EXPECT(pt_set_moe_routes(h, routes_out, nullptr) == PT_OK);

  // sequences of different lengths
  std::vector<int32_t> lens;
  int64_t total = 0;
  for (int b = 0; b < B; ++b) {
    lens.push_back(1 + (b * 37 + 5) % (c.max_seq - 3));
    total += lens.back();
  }
  if (c.n_experts) {
    EXPECT(pt_prefill_ragged(h, V ? tokens : nullptr, V ? nullptr : hidden_in, 1, B, lens.data(), PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_BAD_STATE);
    EXPECT(pt_set_moe_routes(h, nullptr, nullptr) == PT_OK);
  }
  EXPECT(total <= rows + (int64_t)B * c.max_seq);
  int32_t* rtok = (int32_t*)io.get(total * 4, "ragged tokens");
  float* rhid = (float*)io.get((size_t)T * total * d * 4, "ragged hidden in");
  float* rlog = V ? (float*)io.get((size_t)total * V * 4, "ragged logits") : nullptr;
  float* rout = (float*)io.get((size_t)total * d * 4, "ragged hidden out");
  float* rtaps = (float*)io.get((size_t)merges * total * d * 4, "ragged taps");
  float* rttaps = (float*)io.get((size_t)merges * T * total * d * 4, "ragged track taps");
  EXPECT(pt_set_taps(h, rtaps, rttaps) == PT_OK);
  if (V) EXPECT(pt_prefill_ragged(h, rtok, nullptr, 1, B, lens.data(), PT_LOGITS_ALL, rlog, rout) == PT_OK);
  EXPECT(pt_prefill_ragged(h, nullptr, rhid, T, B, lens.data(), V ? PT_LOGITS_LAST : PT_LOGITS_NONE, rlog, rout) == PT_OK);
  EXPECT(pt_set_taps(h, nullptr, nullptr) == PT_OK);
  EXPECT(pt_prefill_ragged(h, nullptr, rhid, 1, B, lens.data(), PT_LOGITS_NONE, nullptr, nullptr) == PT_OK);
  std::vector<int32_t> got(B);
  EXPECT(pt_seq_lens(h, got.data()) == PT_OK && got == lens);
  int32_t longest = 0;
  for (int32_t x : lens) longest = x > longest ? x : longest;
  EXPECT(pt_seq_len(h) == longest);
  while ((rc = pt_decode_step(h, V ? tokens : nullptr, V ? nullptr : hidden_in, 1, B, V ? logits : nullptr, hidden_out, V ? amax : nullptr)) == PT_OK) {}
  EXPECT(rc == PT_ERR_CAPACITY && pt_seq_len(h) == c.max_seq);
  EXPECT(pt_seq_lens(h, got.data()) == PT_OK && got[0] == lens[0] + (c.max_seq - longest));
  lens[0] = 0;
  EXPECT(pt_prefill_ragged(h, nullptr, rhid, 1, B, lens.data(), PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_INVALID_ARGUMENT);
  lens[0] = c.max_seq + 1;
  EXPECT(pt_prefill_ragged(h, nullptr, rhid, 1, B, lens.data(), PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_CAPACITY);
  EXPECT(pt_prefill_ragged(h, nullptr, rhid, 1, B, nullptr, PT_LOGITS_NONE, nullptr, nullptr) == PT_ERR_NULL_POINTER);
  EXPECT(pt_reset(h) == PT_OK && pt_seq_len(h) == 0);
  EXPECT(pt_destroy(h) == PT_OK);
}

int main() {
  invalid_configs();
  // stateless entry points
  {
    io_alloc io;
    const void* tr[16];
    for (int i = 0; i < 16; ++i) tr[i] = io.get(1024 * 64 * 4, "merge track");
    void* out = io.get(1024 * 64 * 4, "merge out");
    EXPECT(pt_track_merge(tr, 16, 1024, 64, PT_F32, 0.5f, out, nullptr) == PT_OK);
    EXPECT(pt_track_merge(tr, 17, 1024, 64, PT_F32, 0.5f, out, nullptr) == PT_ERR_INVALID_ARGUMENT);
    EXPECT(pt_track_merge(tr, 2, 1024, 12, PT_F32, 0.5f, out, nullptr) == PT_ERR_INVALID_ARGUMENT);
    EXPECT(pt_track_merge(nullptr, 2, 1024, 64, PT_F32, 0.5f, out, nullptr) == PT_ERR_NULL_POINTER);
    EXPECT(pt_track_merge(tr, 2, 0, 64, PT_BF16, 1.f, out, nullptr) == PT_OK);
    EXPECT(pt_argmax((const float*)tr[0], 4, 100, (int32_t*)out, nullptr) == PT_OK);
    EXPECT(pt_argmax((const float*)tr[0], -1, 100, (int32_t*)out, nullptr) == PT_ERR_INVALID_ARGUMENT);
  }
  const pt_config models[] = {
      make(2, 4, 2, 128, 4, 4, 32, 512, 512, 2, 64, PT_F32),            // Tiny-like fp32
      make(3, 3, 1, 256, 4, 2, 64, 512, 1024, 5, 200, PT_BF16),         // GQA, three tracks, merge after every layer
      make(2, 2, 2, 512, 4, 1, 128, 1024, 2048, 64, 130, PT_BF16),      // decode GEMMs with K slices, batch 64
      make(4, 2, 1, 512, 8, 8, 64, 1536, 0, 3, 140, PT_BF16),           // hidden states in, hidden states out
      make(1, 3, 1, 256, 4, 4, 64, 512, 1024, 2, 100, PT_BF16),         // one track: the dense twin
      make(2, 2, 1, 512, 4, 2, 128, 512, 1024, 4, 136, PT_BF16, 8, 2),  // PT-MoE
      make(2, 2, 2, 128, 4, 4, 32, 96, 512, 2, 70, PT_F32, 3, 3),       // PT-MoE fp32, every expert taken
      make(2, 2, 2, 256, 4, 4, 64, 256, 512, 48, 72, PT_BF16, 16, 1),   // PT-MoE, more experts than most rows fill
  };
  for (int mode = 0; mode < 2; ++mode)
    for (const pt_config& c : models) run_model(c, mode);
  printf("host_check: %ld launches, %ld buffers checked, all inside their memory\n", hc_launches(), hc_checked());
  return 0;
}

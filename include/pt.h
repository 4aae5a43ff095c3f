/*
 * pt.h - C ABI of the MI355X (gfx950) Parallel Track (PT) transformer forward library.
 *
 * The library computes Algorithm 1 of the paper ("Track Parallelism for PT Transformer",
 * Section 2.2): n independent transformer tracks of L layers each; after every D-th layer the
 * per-track activations are all-reduced and every track continues from the reduced activation.
 * On one GPU all tracks are resident and run as a track-batched prefill and a KV-cached decode;
 * the all-reduce is an on-device reduction (pt_track_merge).
 *
 * The paper does not define the "standard transformer layer" inside a track beyond
 * grouped-query attention (Section 3.1, Table 1).  This library fixes it as: pre-norm RMSNorm,
 * rotary position embedding (rotate-half pairing), causal softmax attention with grouped KV
 * heads, SwiGLU feed-forward, no biases, one shared embedding, one final RMSNorm and an untied
 * output head applied to the merged activation.
 *
 * Conventions
 *  - Every function returns PT_OK (0) or a negative PT_ERR_* code; none throws, aborts or
 *    prints.  pt_last_error() returns a thread-local description of the last failure.
 *  - "dev" pointers are HIP device pointers, "host" pointers are host memory.
 *  - Ownership: the caller allocates every device buffer and the stream and keeps them alive
 *    until pt_destroy; the library never allocates or frees device memory.  It sub-allocates
 *    the three arenas handed to pt_create.
 *  - All device work is enqueued on the stream given to pt_create (pt_track_merge: on the
 *    stream argument) and is asynchronous; the caller synchronises.
 *  - Calls on one handle must not overlap.
 */
#ifndef PT_H_
#define PT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { PT_F32 = 0, PT_BF16 = 1 };

enum {
  PT_OK = 0,
  PT_ERR_INVALID_CONFIG = -1,
  PT_ERR_NULL_POINTER = -2,
  PT_ERR_ARENA_TOO_SMALL = -3,
  PT_ERR_CAPACITY = -4,  /* batch or sequence beyond max_batch / max_seq */
  PT_ERR_BAD_STATE = -5, /* e.g. decode before prefill, forward before weights exist */
  PT_ERR_HIP = -6,
  PT_ERR_INVALID_ARGUMENT = -7
};

/* Which logits pt_prefill writes. */
enum { PT_LOGITS_NONE = 0, PT_LOGITS_LAST = 1, PT_LOGITS_ALL = 2 };

/* Logical tensors of the model, for pt_set_weight / pt_get_weight.  Logical layouts follow
 * the "x @ W" convention, row-major:
 *   WQ [d, H*hd]  WK, WV [d, Hkv*hd]  WO [H*hd, d]  WG, WU [d, f]  WD [f, d]
 *   G1, G2 [d] (RMSNorm gains before attention / before the FFN)
 *   EMBED [vocab, d]  HEAD [d, vocab]  GF [d] (final RMSNorm gain)
 *   ROUTER [d, n_experts] (PT-MoE models only)
 * The numbering of the random tensors equals the stream kinds of the seeded generator.
 * PT-MoE models hold WG, WU, WD once per expert: expert e of layer l is addressed with
 * layer = PT_EXPERT_LAYER(l, e) (also the layer field of that tensor's random stream). */
enum {
  PT_W_EMBED = 1, PT_W_HEAD = 2, PT_W_Q = 3, PT_W_K = 4, PT_W_V = 5, PT_W_O = 6,
  PT_W_G = 7, PT_W_U = 8, PT_W_D = 9, PT_W_G1 = 10, PT_W_G2 = 11, PT_W_GF = 12, PT_W_ROUTER = 13
};
#define PT_EXPERT_LAYER(layer, expert) ((layer) | (((expert) + 1) << 12))

/* Shape of a PT model.  Algorithm 1's n, L, D are n_tracks, n_layers, block_depth; the
 * remaining fields give the per-track layer (Section 3.1: heads and KV heads are per track). */
typedef struct pt_config {
  int32_t n_tracks;    /* n in 1..16 */
  int32_t n_layers;    /* L per track, L % block_depth == 0 */
  int32_t block_depth; /* D: layers between two merges */
  int32_t d_model;     /* per-track width; multiple of 8 */
  int32_t n_heads;     /* query heads per track */
  int32_t n_kv_heads;  /* KV heads per track; divides n_heads */
  int32_t head_dim;    /* multiple of 8 */
  int32_t d_ffn;       /* multiple of 32 */
  int32_t vocab;       /* multiple of 8; 0: hidden-state in, hidden-state out (no embedding, no head) */
  int32_t max_batch;
  int32_t max_seq;     /* KV-cache capacity per sequence */
  int32_t dtype;       /* PT_F32 | PT_BF16: weights, KV cache, GEMM/attention operands.
                          Residual stream, merge, softmax statistics and accumulators are fp32. */
  float merge_scale;   /* merged h = merge_scale * sum_i h_i; 1 = the literal all-reduce sum */
  float rms_eps;
  float rope_theta;
  float init_std;      /* standard deviation used by pt_init_weights */
  /* PT-MoE (Section 2.2 and the Conclusion: MoE sparsity applied inside every track, tracks and merges
   * unchanged).  n_experts = 0: dense SwiGLU feed-forward network.  n_experts = E in 1..64: the network of
   * every (track, layer) is a mixture of E SwiGLU experts of width d_ffn each; a token's router logits are
   * r = RMSNorm(h) W_router, its top_k experts are the largest logits (lowest index on exact ties), their
   * gates the softmax over those top_k logits, and the layer adds sum_e gate_e * expert_e(RMSNorm(h)).
   * No shared expert, no capacity limit (no token is dropped).  n_layers < 4096 for such models. */
  int32_t n_experts;
  int32_t top_k;       /* 1..min(8, n_experts) when n_experts > 0, else 0 */
} pt_config;

typedef struct pt_handle pt_handle;

/* Host only.  Validates cfg and reports the bytes of the three device arenas pt_create needs:
 * weights, KV cache, workspace.  Any out pointer may be NULL. */
int pt_query_bytes(const pt_config* cfg, size_t* weight_bytes, size_t* kv_bytes, size_t* ws_bytes);

/* Creates a handle over caller-owned arenas (256-byte aligned device pointers) and a caller-
 * owned hipStream_t (NULL = the default stream).  Touches no device memory.
 * Errors: INVALID_CONFIG, NULL_POINTER, ARENA_TOO_SMALL. */
int pt_create(const pt_config* cfg, void* dev_weights, size_t weight_bytes, void* dev_kv,
              size_t kv_bytes, void* dev_ws, size_t ws_bytes, void* hip_stream, pt_handle** out);
int pt_destroy(pt_handle* h);

/* Fills every weight on the device from the counter-based generator (stream (seed, kind,
 * track, layer), Box-Muller normals scaled by init_std, rounded to cfg.dtype); gains = 1. */
int pt_init_weights(pt_handle* h, uint64_t seed);

/* Copies one logical tensor between a device fp32 buffer in the logical layout above and the
 * library's physical storage (rounding to cfg.dtype on the way in).  track/layer are ignored
 * for EMBED, HEAD and GF. */
int pt_set_weight(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, const float* dev_src);
int pt_get_weight(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, float* dev_dst);

/* Prefill (Algorithm 1 over B sequences of S tokens starting at position 0; fills the KV cache
 * and sets every sequence length to S).
 *   dev_tokens     int32 [B, S]; used when cfg.vocab > 0 and dev_hidden_in == NULL.
 *   dev_hidden_in  fp32 [hidden_tracks, B*S, d] with hidden_tracks == 1 (the same input x for
 *                  every track, as in Algorithm 1) or == n_tracks (per-track inputs).
 *   logits_mode    PT_LOGITS_*; dev_logits fp32 [B, V] (LAST) or [B*S, V] (ALL); needs vocab > 0.
 *   dev_hidden_out fp32 [B*S, d], the output activation h of Algorithm 1; may be NULL.
 * Errors: NULL_POINTER, CAPACITY (B > max_batch or S > max_seq), BAD_STATE, INVALID_ARGUMENT. */
int pt_prefill(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
               int32_t hidden_tracks, int32_t B, int32_t S, int32_t logits_mode,
               float* dev_logits, float* dev_hidden_out);

/* Prefill of a batch of sequences of different lengths (the throughput mode of Section 3.3, Tables 5 and 8:
 * large batches of mixed input lengths).  Sequence b has host_lens[b] tokens, 1 <= host_lens[b] <= max_seq
 * (host_lens is a HOST array of B entries).  Inputs and outputs are packed, sequence after sequence, without
 * padding; n = host_lens[0] + ... + host_lens[B-1]:
 *   dev_tokens     int32 [n]; or dev_hidden_in fp32 [hidden_tracks, n, d]
 *   dev_logits     fp32 [B, V] (PT_LOGITS_LAST: each sequence's own last token) or [n, V] (PT_LOGITS_ALL)
 *   dev_hidden_out fp32 [n, d]
 *   taps set by pt_set_taps hold rows = n packed rows per merge.
 * Every sequence sees only its own tokens (positions 0 .. len-1, causal).  Afterwards pt_decode_step appends
 * one token to every sequence at that sequence's own position; pt_seq_lens reports the lengths and pt_seq_len
 * the longest.  Inside, each sequence is padded to a multiple of 64 rows with zero-vector rows that run
 * through the layers like appended tokens (the causal mask keeps them from every real position); their cache
 * entries are overwritten by the decode steps that reach those positions.
 * Errors as pt_prefill; INVALID_ARGUMENT for a length below 1, CAPACITY for one above max_seq. */
int pt_prefill_ragged(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in, int32_t hidden_tracks,
                      int32_t B, const int32_t* host_lens, int32_t logits_mode, float* dev_logits,
                      float* dev_hidden_out);

/* One KV-cached decode step: one new row per sequence at position len, appended to the cache.
 *   dev_tokens int32 [B] or dev_hidden_in fp32 [hidden_tracks, B, d]; B must equal the B of the
 *   preceding prefill.  After pt_prefill_ragged every sequence continues at its own length.  dev_logits fp32 [B, V], dev_hidden_out fp32 [B, d], dev_argmax int32 [B]
 *   (lowest id on ties); dev_logits and dev_hidden_out may each be NULL; dev_argmax may be NULL
 *   and, when given, needs dev_logits as well (the ids are taken from the stored logits).
 * Errors as pt_prefill; CAPACITY when len + 1 > max_seq; BAD_STATE before a prefill;
 * NULL_POINTER for dev_argmax without dev_logits. */
int pt_decode_step(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                   int32_t hidden_tracks, int32_t B, float* dev_logits, float* dev_hidden_out,
                   int32_t* dev_argmax);

/* pt_decode_step for callers that cannot allocate device memory or reserve a workspace for decoding: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors as pt_decode_step, but every temporary of the step (residual streams, normed activations, q, attention
 * output, SwiGLU product, decode-attention split partials, K slices of the decode GEMMs) lives in a static
 * device array inside the library (32 MiB per GPU, held from library load to process end) instead of the
 * workspace arena given to pt_create; only the weight and KV arenas of the handle and the caller's input and
 * output buffers are touched besides.  Calls no hipMalloc / hipFree or any allocating routine.
 *   Limit: the temporaries of one step at batch B must fit the array, else PT_ERR_CAPACITY and nothing is
 *   launched (examples that fit: Mid PT at batch 32, Large PT at batch 64, the one-GPU share at batch 64).
 *   All calls on one GPU share that GPU's array, whatever the handle: calls that overlap in time on one GPU
 *   (different streams or threads) race.  The array keeps the previous call's contents; nothing in it needs to
 *   start at zero, every kernel writes what it later reads. */
int pt_decode_step_static(pt_handle* h, const int32_t* dev_tokens, const float* dev_hidden_in,
                          int32_t hidden_tracks, int32_t B, float* dev_logits, float* dev_hidden_out,
                          int32_t* dev_argmax);

/* The track merge of Algorithm 1 (the all-reduce, as an on-device reduction), stateless:
 *   out[t, :] = scale * (tracks[0][t, :] + ... + tracks[n-1][t, :]), fp32 accumulation in track
 *   order, for t < tokens.  host_tracks is a HOST array of n DEVICE pointers, each [tokens, d]
 *   of element type dtype (PT_F32 | PT_BF16); dev_out has the same type and may alias
 *   tracks[0].  n <= 16.  d must be a multiple of 8.  Enqueued on hip_stream. */
int pt_track_merge(const void* const* host_tracks, int32_t n, int64_t tokens, int32_t d,
                   int32_t dtype, float scale, void* dev_out, void* hip_stream);

/* Greedy token choice, stateless: dev_out[r] = index of the largest of dev_logits[r, 0..vocab), the
 * lowest index on exact ties (the rule both sides of the parity tests use); fp32 logits [rows, vocab]
 * row-major, int32 out [rows].  The same kernel serves dev_argmax of pt_decode_step.  Enqueued on
 * hip_stream.  Errors: NULL_POINTER, INVALID_ARGUMENT (rows < 0 or vocab < 1). */
int pt_argmax(const float* dev_logits, int32_t rows, int32_t vocab, int32_t* dev_out, void* hip_stream);

/* Optional observation point: when set (non-NULL), every merge inside pt_prefill /
 * pt_decode_step also stores the merged activation to dev_taps, fp32
 * [n_layers / block_depth, rows, d] with rows = B*S (prefill) or B (decode), and the per-track
 * activations right before the merge to dev_track_taps (may be NULL), fp32
 * [n_layers / block_depth, n_tracks, rows, d]. */
int pt_set_taps(pt_handle* h, float* dev_taps, float* dev_track_taps);

/* PT-MoE observation / forcing point for the expert selection (both may be NULL = off), int32
 * [n_layers, n_tracks, rows, top_k] with rows as for pt_set_taps, experts in decreasing order of logit:
 * dev_routes_out receives the selection every forward call makes; dev_routes_in prescribes it (the gates
 * stay the softmax of the router's own logits at the prescribed experts; entries must be distinct and in
 * [0, n_experts), else bit 1 of the status word checked by pt_sync_status is raised and expert 0.. are used).
 * The selection is an integer decided by floating point, so a caller that compares two implementations
 * forces one's selection on the other.  Not available with pt_prefill_ragged (BAD_STATE from that call).
 * Errors: NULL_POINTER (handle), BAD_STATE (dense model). */
int pt_set_moe_routes(pt_handle* h, int32_t* dev_routes_out, const int32_t* dev_routes_in);

/* Kernel selection.  PT_PATH_AUTO (default) uses the MFMA / bandwidth-tuned kernels wherever the
 * shape allows and the shape-generic kernels elsewhere; PT_PATH_GENERIC forces the shape-generic
 * kernels everywhere (slow; used to cross-check the tuned kernels). */
enum { PT_PATH_AUTO = 0, PT_PATH_GENERIC = 1 };
int pt_set_kernel_path(pt_handle* h, int32_t path);

/* Token ids outside [0, vocab) are not an error the asynchronous forward calls can return: the
 * embedding kernel reads row 0 (negative ids) or row vocab-1 instead and raises a flag in device
 * memory.  pt_sync_status synchronises the handle's stream, reads and clears that flag and returns
 * PT_ERR_INVALID_ARGUMENT if any forward call since the previous pt_sync_status (or pt_create) met
 * such an id; the logits of those calls are then meaningless.  PT_OK otherwise. */
int pt_sync_status(pt_handle* h);

/* Forgets all sequences (lengths = 0); the KV cache contents become dead. */
int pt_reset(pt_handle* h);

/* Number of merges executed by forward calls on this handle since pt_create (one per track
 * block: L/D per forward pass, against 2L sync points of tensor parallelism; Section 2.2). */
int64_t pt_merge_count(const pt_handle* h);

/* Current sequence length (after pt_prefill: identical for all sequences; after pt_prefill_ragged: the
 * longest), or a negative error. */
int32_t pt_seq_len(const pt_handle* h);
/* Writes the current length of every live sequence to host_out (HOST array of at least B entries). */
int pt_seq_lens(const pt_handle* h, int32_t* host_out);

/* Per-kernel timing with HIP events on the handle's stream.  Kernel classes: */
enum {
  PT_K_EMBED = 0, PT_K_RMSNORM = 1, PT_K_GEMM_QKV = 2, PT_K_ATTN_PREFILL = 3, PT_K_ATTN_DECODE = 4,
  PT_K_GEMM_OUT = 5, PT_K_GEMM_GATEUP = 6, PT_K_GEMM_DOWN = 7, PT_K_MERGE = 8, PT_K_GEMM_HEAD = 9,
  PT_K_OTHER = 10,
  PT_K_GEMM_ROUTER = 11, /* PT-MoE: router logits */
  PT_K_MOE = 12,         /* PT-MoE: expert selection, grouping of tokens by expert, weighted combine */
  PT_K_COUNT = 13
};
/* class_mask: bit k set = bracket every launch of class k in later forward calls with a pair of
 * events (0 switches timing off).  Each bracketed launch costs two event records on the stream. */
int pt_profile_enable(pt_handle* h, uint32_t class_mask);
/* Synchronises the stream, folds all finished event pairs into the totals and returns, for one
 * class, the summed kernel time in milliseconds and the number of launches since the last
 * pt_profile_reset.  Either out pointer may be NULL. */
int pt_profile_read(pt_handle* h, int32_t kernel_class, double* total_ms, int64_t* launches);
int pt_profile_reset(pt_handle* h);

/* Which kernel family served the launches of a class (counted on the host at every launch of a
 * GEMM or attention class, whether or not timing is on; zeroed by pt_profile_reset).  Family 0 is
 * the shape-generic kernel that takes whatever the tuned ones refuse, so a test can tell a tuned
 * launch from a silent fall-back:
 *   GEMM classes       1 = MFMA tile kernel (more than 64 rows), 2 = weight-streaming kernel
 *                      (5..64 rows), 3 = matrix-vector kernel (1..4 rows)
 *   PT_K_ATTN_PREFILL  1 = flash-style kernel with LDS key/value tiles, 2 = its register-operand
 *                      form (lengths that are a multiple of 32 but not of 64)
 *   PT_K_ATTN_DECODE   1 = matrix-core split-K kernel (up to 32 query heads per KV head),
 *                      2 = vector split-K kernel (larger groups)
 * counts receives PT_FAMILY_COUNT values. */
enum { PT_FAMILY_GENERIC = 0, PT_FAMILY_COUNT = 4 };
int pt_profile_paths(pt_handle* h, int32_t kernel_class, int64_t* counts);

/* Process-wide tuning overrides for benchmark sweeps; the defaults select by shape.
 *   PT_TUNE_GEMM_TILE_CONFIG   value -1 (default): automatic; 0..11: force that tile configuration
 *                              of the MFMA GEMM wherever it fits the shape
 *   PT_TUNE_SKINNY_PLAN        value 0 (default): automatic; else 256 * workgroups per track +
 *                              K slices for the weight-streaming GEMM (where the shape allows)
 *   PT_TUNE_FOLD_RMSNORM       value 1 (default): in prefill the RMSNorm between two GEMMs is folded into
 *                              them (scaled bf16 copy and row sums from the producer's epilogue, row factor in
 *                              the consumer's); 0: a separate RMSNorm kernel runs instead
 *   PT_TUNE_ATTN_PREFILL       value 0 (default): the LDS-tiled flash prefill kernel; 1: its software-pipelined
 *                              form (8 wavefronts per workgroup, four direct-to-LDS stages, softmax slices
 *                              interleaved with the MFMAs; measured slower, kept for comparison)
 * Not thread-safe against concurrent forward calls.  Errors: INVALID_ARGUMENT (unknown knob). */
enum { PT_TUNE_GEMM_TILE_CONFIG = 0, PT_TUNE_SKINNY_PLAN = 1, PT_TUNE_FOLD_RMSNORM = 2, PT_TUNE_ATTN_PREFILL = 3 };
int pt_set_tuning(int32_t knob, int32_t value);

const char* pt_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PT_H_ */

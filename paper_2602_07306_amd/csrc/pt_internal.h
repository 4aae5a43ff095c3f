// Internal declarations shared by the host-side API and the HIP kernels of libpt.
#ifndef PT_INTERNAL_H_
#define PT_INTERNAL_H_

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

// The library is built with hidden symbol visibility; only what pt.h declares is exported.
#pragma GCC visibility push(default)
#include "pt.h"
#pragma GCC visibility pop

typedef uint16_t bf16_t;  // raw bfloat16 bits

// ---------------------------------------------------------------------------------------------
// Physical storage (chosen for gfx950; the logical "x @ W" layouts are in pt.h).
//
// Every GEMM weight is stored transposed, [N, K] with K contiguous, so that both MFMA operands
// are read along the contraction dimension:
//   wqkv [(H + 2*Hkv)*hd, d]   rows: all q columns, then all k columns, then all v columns
//   wo   [d, H*hd]
//   wgu  [2f, d]               gate and up interleaved in blocks of 32 rows:
//                              row (j/32)*64 + j%32 = gate_j, row (j/32)*64 + 32 + j%32 = up_j,
//                              so a 32-column MFMA tile of gate sits next to the same tile of up
//   wd   [d, f]
//   embed [V, d], headT [V, d]
// KV cache, per (track, layer, sequence, kv head):
//   K  [max_seq, hd]   (hd contiguous: the contraction dimension of q.k)
//   Vt [hd, s_pad]     (positions contiguous: the contraction dimension of p.v), row pitch s_pad
//                      = max_seq rounded up to 64, plus 64 so that rows do not alias HBM channels.
// ---------------------------------------------------------------------------------------------
struct pt_layout {
  // element counts
  int64_t n_qkv;        // (H + 2*Hkv) * hd
  int64_t hq;           // H * hd
  int64_t hk;           // Hkv * hd
  int64_t wqkv_elems, wo_elems, wgu_elems, wd_elems;  // per (track, layer); gate/up and down once per expert
  int64_t wr_elems;                                    // PT-MoE router [e_pad, d] (0 for a dense model)
  int64_t e_pad;                                       // experts rounded up to 4: pitch of the router logits
  int64_t expert_elems;                                // wgu_elems + wd_elems: distance between two experts
  int64_t off_wr_elems, off_exp_elems;                 // element offsets of the router / first expert in a layer block
  int64_t layer_w_elems;                               // everything of one (track, layer)
  int64_t s_pad;                                       // Vt row pitch (elements)
  // byte offsets inside the weight arena
  size_t off_layers;    // [T][L] blocks of layer_w_elems elements
  size_t off_gains;     // fp32 [T][L][2][d]
  size_t off_gf;        // fp32 [d]
  size_t off_embed;     // dtype [V, d]
  size_t off_headT;     // dtype [V, d]
  size_t off_rope;      // fp32 [max_seq, hd/2, 2] cos, sin (a constant of the model, written by the first forward call)
  size_t off_flag;      // int32 device status word (bit 0: a token id was out of range)
  size_t weight_bytes;
  // KV arena
  int64_t kv_seq_elems;  // per (t, l, b, hkv): max_seq*hd (K) ; hd*s_pad (Vt)
  size_t off_k, off_v, off_seq, kv_bytes;   // off_seq: int4 [max_batch] per-sequence state of a ragged batch
  int64_t s_k;                              // K rows per head and rotary-table rows: max_seq rounded up to 64
  size_t ws_bytes;    // workspace arena: a pt_workspace for M = max_batch * max_seq rows
  int32_t elem_size;  // 4 or 2
};

// Temporaries of one forward call over `rows` rows per track, as offsets into one block of device memory: the
// caller's workspace arena (sized for max_batch * max_seq rows) or, for pt_decode_step_static, the library's
// static device array (sized for the rows of that call).
struct pt_workspace {
  char* base;
  size_t off_h;       // fp32 [T, rows, d] residual streams
  size_t off_hm;      // fp32 [rows, d]    merged activation
  size_t off_a;       // dtype [T, rows, d] normed activations
  size_t off_q;       // dtype [T, rows, hq]
  size_t off_o;       // dtype [T, rows, hq] attention output
  size_t off_m;       // dtype [T, rows, f]  SwiGLU product
  size_t off_part;    // fp32 split-K decode-attention partials, [T*B*H][max_splits][hd + 2]
  size_t off_skp;     // fp32 K slices of the decode residual GEMMs, [slice][T][rows][d]
  size_t off_ss;      // fp32 [T, rows, d / 64] per-row partial sums of squares (RMSNorm folded into the GEMMs)
  size_t off_rinv;    // fp32 [T, rows] 1/rms of every row, from those sums
  size_t off_rowmap;  // int2 [rows] (sequence, position) of every row of a ragged batch
  size_t off_rowidx;  // int32 [rows] packed row of every valid token, then [max_batch] last rows (ragged prefill)
  // PT-MoE (all absent for a dense model).  An assignment is one (row, chosen expert) pair; assignments are
  // grouped by expert into `slots`: expert e of a track owns a segment of slots that starts at a multiple of 256.
  int64_t slots;      // slot capacity per track: rows * top_k plus up to 255 padding slots per expert, a multiple of 256
  size_t off_rlogit;  // fp32 [T, rows, e_pad] router logits
  size_t off_route;   // int32 [T, rows, k] chosen experts
  size_t off_gate;    // fp32 [T, rows, k] their gates
  size_t off_slot;    // int32 [T, rows, k] slot of every assignment
  size_t off_perm;    // int32 [T, slots] row of every slot (some valid row in padding slots)
  size_t off_blk;     // int32 [T, slots / 64] expert of every 64-slot block, -1 where the block holds no assignment
  size_t off_cnt;     // int32 [T, rows / 256 + 2, 64] per 256-row block: assignments per expert in earlier blocks; then totals, segment bases
  size_t off_y;       // fp32 [T, slots, d] expert outputs per slot
  size_t bytes;
  int64_t skp_floats; // capacity behind off_skp
  int32_t max_splits; // capacity behind off_part, in splits per (track, sequence, head)
};

struct pt_prof_pair {
  int cls;
  hipEvent_t e0, e1;
};

struct pt_prof {
  uint32_t mask = 0;
  std::vector<hipEvent_t> free_events;
  std::vector<pt_prof_pair> pending;
  double ms[PT_K_COUNT] = {0};
  int64_t launches[PT_K_COUNT] = {0};
  int64_t family[PT_K_COUNT][PT_FAMILY_COUNT] = {{0}};   // launches per kernel family (see pt_profile_paths)
};

// Per-sequence state of a ragged batch, on the host; the device copy (int4 per sequence: first row of the
// padded-packed prefill layout, padded length, length, first token of the packed input) sits at the end of the
// KV arena.
struct pt_seq {
  int32_t row0, plen, len, tok0;
};

struct pt_handle {
  pt_config cfg;
  pt_layout lay;
  char* w;
  char* kv;
  char* ws;
  pt_workspace arena;           // the caller's workspace arena, laid out for max_batch * max_seq rows
  const pt_workspace* active;   // temporaries of the forward call in progress
  hipStream_t stream;
  int32_t batch;      // B of the live sequences (0: none)
  int32_t seq_len;    // their common length (the longest one when ragged)
  bool ragged;        // the live sequences came from pt_prefill_ragged: per-sequence lengths in seqs / on the device
  std::vector<pt_seq> seqs;
  int64_t merges;
  bool weights_ready;
  bool rope_ready;    // the rotary table and the device status word have been written
  float* taps;
  float* track_taps;
  int32_t* routes_out;          // PT-MoE observation / forcing points (pt_set_moe_routes)
  const int32_t* routes_in;
  int32_t path;
  pt_prof prof;
};

int pt_set_error(int code, const char* fmt, ...);
int pt_validate_config(const pt_config* c);
int pt_compute_layout(const pt_config* c, pt_layout* l);
// Lays out the temporaries of a forward call over `rows` rows per track (`batch` sequences) from offset 0;
// skp_floats and max_splits are the capacities wanted for the two split scratch areas.
void pt_layout_workspace(const pt_config* c, const pt_layout* l, int64_t rows, int64_t batch, int64_t skp_floats,
                         int32_t max_splits, pt_workspace* w);

// ---------------------------------------------------------------------------------------------
// GEMM: C[b] (M x N) = A[b] (M x K, row-major, lda) * W[b]^T, W[b] is [N, K] row-major (ldb),
// for b < batch (the track dimension), followed by one of the fused epilogues.
// ---------------------------------------------------------------------------------------------
enum { EPI_STORE_F32 = 0, EPI_RESIDUAL = 1, EPI_SWIGLU = 2, EPI_QKV = 3 };

struct pt_gemm_args {
  const void* A;
  const void* W;
  int64_t a_bstride, w_bstride;  // elements between tracks
  int32_t lda, ldb;
  int32_t M, N, K, batch;
  int32_t dtype;                 // operand type
  int32_t epi;
  // EPI_STORE_F32: out[b][m][n] = acc                       (out_bstride, ldo)
  // EPI_RESIDUAL : out[b][m][n] = res[b][m][n] + acc         (res may alias out; res_bstride may be 0)
  float* out;
  const float* res;
  int64_t out_bstride, res_bstride;
  int32_t ldo;
  // EPI_SWIGLU   : olp[b][m][j] = silu(gate_j) * up_j, N = 2f in the interleaved order, ld = N/2
  void* olp;
  int64_t olp_bstride;
  // EPI_QKV      : RoPE on q and k columns; q -> olp [b][m][hq]; k, v -> the KV cache.
  //                Row m is token (m / S) at position pos0 + m % S.
  void* kc;
  void* vc;
  const float* rope;             // [max_seq][hd/2][2]
  // cache head index = track * kv_bstride + sequence * kv_seq_stride + kv head; a head holds
  // kv_head_elems = max_seq * hd elements of K and hd * s_pad elements of V^T
  int64_t kv_bstride, kv_seq_stride, kv_head_elems;
  int32_t H, Hkv, hd, S, pos0, s_pad;
  // Ragged batches (sequences of different lengths): when row_map is given, row m belongs to sequence
  // row_map[m].x at position row_map[m].y instead of (m / S, pos0 + m % S).  row_blocks != 0 promises that
  // every aligned block of 32 rows lies in one sequence at consecutive positions starting at a multiple of 32
  // (the padded-packed layout of a ragged prefill), which the LDS-staged QKV epilogue relies on.
  const int2* row_map;
  int32_t row_blocks;
  // K-slice scratch of the decode kernel, sk_part_floats floats (may be null: K is not split over workgroups)
  float* sk_part;
  int64_t sk_part_floats;
  // Optional, honoured only where pt_gemm_fuses_norm(g) holds: A is not read; row m of track b is
  // RMSNorm(norm_src[b][m][0..K)) * norm_gain[b][0..K), formed by the kernel itself.
  const float* norm_src;
  const float* norm_gain;
  int64_t norm_bstride, norm_gbstride;
  float norm_eps;
  // RMSNorm folded into the two GEMMs around it (MFMA tile kernels only, see pt_gemm_mfma_fold_parts).
  //   producer, EPI_RESIDUAL: besides out, the kernel stores bf16(out[b][m][n] * nf_gain[b][n]) to nf_out [b][m][N]
  //   and, per row, the sum of out^2 over each block of N / nf_parts columns to nf_ss[b][m][part];
  //   pt_launch_row_inv_rms turns the partial sums into one factor 1 / sqrt(mean(out^2) + eps) per row;
  //   consumer, EPI_QKV / EPI_SWIGLU: the accumulators of row m are multiplied by rs_inv[b][m] before the
  //   epilogue (A then holds bf16(h * gain), unnormalised).
  void* nf_out;
  const float* nf_gain;
  float* nf_ss;
  int64_t nf_out_bstride, nf_gain_bstride, nf_ss_bstride;
  int32_t nf_parts;
  const float* rs_inv;
  int64_t rs_bstride;
  // Grouped GEMM (PT-MoE experts): rows are slots grouped by expert in 256-aligned segments.
  //   a_rows    : when given, GEMM row m of track b reads A row a_rows[b * a_rows_bstride + m] (a gather)
  //   blk_group : per 64-row block of track b, the weight group (expert) of its rows, or -1: the block holds no
  //               row and tiles that start in it do nothing; W of group e starts w_gstride elements after e-1's
  const int32_t* a_rows;
  int64_t a_rows_bstride;
  const int32_t* blk_group;
  int64_t grp_bstride, w_gstride;
  int32_t grp_rows;   // rows an average group holds (a hint for the tile height; 0 = unknown)
  // The same groups as (first row, row count) per group, for the weight-streaming kernel, which takes a whole
  // group per workgroup when no group can hold more than 64 rows (grp_max_rows): group e of track b has
  // grp_count[b * grp_info_bstride + e] rows starting at row grp_base[b * grp_info_bstride + e].
  const int32_t* grp_count;
  const int32_t* grp_base;
  int64_t grp_info_bstride;
  int32_t n_groups, grp_max_rows;
};

enum { PT_SK_PART_FLOATS = 16 << 20 };   // K-slice scratch inside the caller's workspace arena
enum { PT_MAX_SPLITS = 32 };
enum { PT_STATIC_SCRATCH_BYTES = 32 << 20 };   // the static device array behind pt_decode_step_static             // decode-attention splits per (track, sequence, head)

int pt_launch_gemm_generic(const pt_gemm_args& g, hipStream_t s);
// Tuned launchers return 0 if they do not cover the problem (nothing launched), a negative PT_ERR_* code,
// or the kernel family that was launched (the numbering of pt_profile_paths).
// MFMA tile kernels: returns 1 when launched.
int pt_launch_gemm_mfma(const pt_gemm_args& g, hipStream_t s);
// For a residual GEMM that the MFMA tile kernels would run with an LDS-staged epilogue: the number of column
// blocks per row whose sums of squares the kernel can emit (nf_parts), else 0.  Shape fields only.
int pt_gemm_mfma_fold_parts(const pt_gemm_args& g);
// True if the MFMA tile kernels cover the problem (shape fields only).
bool pt_gemm_mfma_covers(const pt_gemm_args& g);
// Weight-streaming kernel for M <= 64 (decode): returns 2, or 3 for its matrix-vector form (M <= 4).  With
// allow_split a residual GEMM may leave pt_gemm_skinny_ksplit(g) > 1 K slices in g.sk_part
// ([slice][batch][M][N] fp32) instead of writing out = res + product; pt_launch_resnorm adds them up.
int pt_launch_gemm_skinny(const pt_gemm_args& g, bool allow_split, hipStream_t s);
int pt_gemm_skinny_ksplit(const pt_gemm_args& g);
// True if pt_launch_gemm_skinny would run this problem (shape fields only) on the kernel that can form its A
// operand from the fp32 residual stream (norm_* fields), which saves the RMSNorm launch in front of it.
bool pt_gemm_fuses_norm(const pt_gemm_args& g);

// ---------------------------------------------------------------------------------------------
// Attention over the KV cache.  q/o: [batch_t][rows][H*hd]; row m is sequence m / S at position
// pos0 + m % S and sees cache positions <= its own.
// ---------------------------------------------------------------------------------------------
struct pt_attn_args {
  const void* q;
  void* o;
  const void* kc;
  const void* vc;
  int64_t q_bstride;             // elements between tracks in q / o
  int64_t kv_bstride, kv_seq_stride, kv_head_elems;
  int32_t n_tracks, B, S, pos0;
  int32_t H, Hkv, hd, s_pad;
  int32_t dtype;
  float* partials;               // split-K workspace (decode)
  int32_t max_splits;
  // Ragged batches.  Decode (S == 1): row_map[seq].y is the position of the new row of sequence seq (its cache
  // holds that many older positions); max_pos is the largest of them.  Prefill: seq_info[seq] = (first row,
  // padded length, length, first token) of the padded-packed layout, rows holds their total and max_plen the
  // longest padded length; row m of q / o is packed row m.
  const int2* row_map;
  const int4* seq_info;
  int32_t max_pos, max_plen;
  int64_t rows;
};

int pt_launch_attn_generic(const pt_attn_args& a, hipStream_t s);
int pt_launch_attn_prefill_mfma(const pt_attn_args& a, hipStream_t s);  // 1: LDS-tiled, 2: register operands
int pt_launch_attn_decode(const pt_attn_args& a, hipStream_t s);        // 1: matrix-core kernel, 2: vector kernel

// Tuning overrides (pt_set_tuning): tile configuration of the MFMA GEMM (-1 = by shape) and plan of the
// weight-streaming GEMM (0 = by shape).
extern int pt_tune_gemm_cfg;
extern int pt_tune_skinny_plan;
extern int pt_tune_attn_prefill;   // 0: plain LDS-tiled flash kernel, 1: software-pipelined flash kernel

// ---------------------------------------------------------------------------------------------
// Elementwise / bandwidth-bound kernels.
// ---------------------------------------------------------------------------------------------
// flag: device status word; bit 0 is set when a token id lies outside [0, vocab)
int pt_launch_embed(const void* embed, int32_t dtype, const int32_t* tokens, int64_t rows, int32_t d,
                    int32_t vocab, float* h, int32_t* flag, hipStream_t s);
// Ragged prefill: packed row r of sequence (row_map[r].x) at position p takes token tokens[tok0 + p] when p <
// len, else the zero vector (padding rows).
int pt_launch_embed_ragged(const void* embed, int32_t dtype, const int32_t* tokens, const int2* row_map,
                           const int4* seq_info, int64_t rows, int32_t d, int32_t vocab, float* h, int32_t* flag,
                           hipStream_t s);
// dst[t][r][:] = (position < length) ? src[t][tok0 + position][:] : 0 over the padded-packed rows (hidden-state input)
int pt_launch_scatter_rows(const float* src, int64_t src_bstride, const int2* row_map, const int4* seq_info,
                           int64_t rows, int32_t d, int32_t batch, float* dst, int64_t dst_bstride, hipStream_t s);
// dst[i][:] = src[idx[i]][:] for i < n (fp32 rows of d elements)
int pt_launch_gather_rows(const float* src, const int32_t* idx, int64_t n, int32_t d, float* dst, hipStream_t s);
// Bookkeeping of a ragged batch from seq_info [B]: row_map [rows] of the padded-packed prefill layout, valid [sum
// of lengths] (packed row of every real token, in input order) and last [B] (packed row of each last token).
int pt_launch_ragged_maps(const int4* seq_info, int32_t B, int64_t rows, int2* row_map, int32_t* valid, int32_t* last,
                          hipStream_t s);
// Decode step of a ragged batch: row_map[b] = (b, length of b); with advance the lengths grow by one afterwards.
int pt_launch_decode_rowmap(int4* seq_info, int32_t B, int2* row_map, hipStream_t s);
int pt_launch_advance_lens(int4* seq_info, int32_t B, hipStream_t s);
int pt_launch_rmsnorm(const float* h, int64_t h_bstride, const float* gains, int64_t g_bstride,
                      void* out, int64_t out_bstride, int32_t dtype, int32_t batch, int64_t rows,
                      int32_t d, float eps, hipStream_t s);
// rows selected by index: out[r] = norm(h[row_index(r)]), row_index(r) = row_idx ? row_idx[r] : r * row_step + row_off
int pt_launch_rmsnorm_rows(const float* h, const float* gain, void* out, int32_t dtype, int64_t rows,
                           int64_t row_step, int64_t row_off, const int32_t* row_idx, int32_t d, float eps, hipStream_t s);
int pt_launch_merge(const void* const* tracks, int32_t n, int64_t elems, int32_t dtype, float scale,
                    void* out, float* tap, hipStream_t s);
int pt_launch_copy_f32(const float* src, float* dst, int64_t elems, hipStream_t s);
int pt_launch_argmax(const float* logits, int32_t rows, int32_t vocab, int32_t* out, hipStream_t s);
int pt_launch_rope_table(float* table, int32_t max_seq, int32_t hd, float theta, hipStream_t s);
// h[b][r][:] = res[b][r][:] + sum over slices of part[slice][b][r][:]  (slices added in order), then, when out
// is given, out[b][r][:] = RMSNorm(h[b][r][:]) * gains[b][:].  res may alias h.  d <= 8192, bf16 out.
int pt_launch_resnorm(const float* part, int32_t slices, const float* res, int64_t res_bstride, float* h,
                      int64_t h_bstride, const float* gains, int64_t g_bstride, void* out, int64_t out_bstride,
                      int32_t batch, int64_t rows, int32_t d, float eps, hipStream_t s);
int pt_launch_fill_f32(float* dst, int64_t n, float v, hipStream_t s);
// out[r] = 1 / sqrt(sum_p ss[r][p] / d + eps) for r < rows (rows of all tracks back to back)
int pt_launch_row_inv_rms(const float* ss, int32_t parts, int64_t rows, int32_t d, float eps, float* out, hipStream_t s);
// ---------------------------------------------------------------------------------------------
// PT-MoE: expert selection, grouping, weighted combine (kernels_moe.hip).  Shapes: T tracks, rows per track, E
// experts (logit pitch e_pad), k experts per row.
// ---------------------------------------------------------------------------------------------
struct pt_moe_args {
  int32_t T, E, e_pad, k;
  int64_t rows, slots;
  const float* logits;   // [T, rows, e_pad]
  int32_t* route;        // [T, rows, k]
  float* gate;           // [T, rows, k]
  int32_t* slot;         // [T, rows, k]
  int32_t* perm;         // [T, slots]
  int32_t* blk;          // [T, slots / 64]
  int32_t* cnt;          // [T, rows / 256 + 2, 64]
  const int32_t* forced; // [T, rows, k] or null; track stride forced_bstride
  int32_t* chosen_out;   // [T, rows, k] or null; same stride
  int64_t obs_bstride;
  int32_t* flag;         // device status word (bit 1: a forced selection was invalid)
};
// Top-k of the router logits and the gates (softmax over the chosen logits), then the grouping: slot of every
// assignment, row of every slot, expert of every 64-slot block.
int pt_launch_moe_route(const pt_moe_args& a, hipStream_t s);
// h[t][r][:] = res[t][r][:] + sum_j gate[t][r][j] * y[t][slot[t][r][j]][:] (j in order), then, when out is given,
// out[t][r][:] = RMSNorm(h[t][r][:]) * gains[t][:] in `dtype`.  res may alias h.
int pt_launch_moe_combine(const pt_moe_args& a, const float* y, const float* res, int64_t res_bstride, float* h,
                          int32_t d, const float* gains, int64_t g_bstride, void* out, int32_t dtype, float eps,
                          hipStream_t s);

// Sets attribute hipFuncAttributeMaxDynamicSharedMemorySize once per kernel (thread-safe: the result is the
// initialiser of a function-local static at the call site).
#define PT_SET_MAX_LDS_ONCE(kern, bytes)                                                                   \
  do {                                                                                                     \
    static const hipError_t attr_rc_ =                                                                     \
        hipFuncSetAttribute((const void*)(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes)); \
    if (attr_rc_ != hipSuccess)                                                                            \
      return pt_set_error(PT_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(attr_rc_));             \
  } while (0)
// weight access: tensor ids are PT_W_*; phys points at the tensor's physical base
int pt_launch_weight_init(pt_handle* h, uint64_t seed);
int pt_launch_weight_copy(pt_handle* h, int32_t tensor, int32_t track, int32_t layer, float* logical,
                          bool to_device_storage);

#define PT_HIP_CHECK(expr)                                                             \
  do {                                                                                 \
    hipError_t e_ = (expr);                                                            \
    if (e_ != hipSuccess) return pt_set_error(PT_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

#endif  // PT_INTERNAL_H_

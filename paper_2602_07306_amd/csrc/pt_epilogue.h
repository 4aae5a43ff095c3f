// Fused GEMM epilogues, stated per pair of output columns.  Both GEMM kernel families call these.
//
// A "pair" is the two accumulators one epilogue step needs together:
//   STORE_F32 / RESIDUAL : any two columns (handled independently)
//   SWIGLU               : (gate_j, up_j) -> silu(gate_j) * up_j
//   QKV                  : q and k sections: (u_j, u_{j+hd/2}) of one head, rotated by the rotary
//                          angle of the row's position (rotate-half pairing); v section: two
//                          independent columns, stored transposed into the V^T cache.
#ifndef PT_EPILOGUE_H_
#define PT_EPILOGUE_H_

#include "pt_device.h"

// (sequence, position) of GEMM row m: by the row map of a ragged batch, else m / S and pos0 + m % S
struct pt_rowpos {
  int seq, pos;
};
__device__ __forceinline__ pt_rowpos gemm_row_pos(const pt_gemm_args& g, int m) {
  if (g.row_map) {
    const int2 e = g.row_map[m];
    return {e.x, e.y};
  }
  const int seq = m / g.S;
  return {seq, g.pos0 + (m - seq * g.S)};
}

// gate/up physical rows sit in 64-row groups: 32 gate rows then the 32 matching up rows
__device__ __forceinline__ int swiglu_gate_row(int j) { return (j >> 5) * 64 + (j & 31); }

template <typename T>
__device__ __forceinline__ void epi_store_f32(const pt_gemm_args& g, int b, int m, int n, float acc) {
  g.out[b * g.out_bstride + (int64_t)m * g.ldo + n] = acc;
}

template <typename T>
__device__ __forceinline__ void epi_residual(const pt_gemm_args& g, int b, int m, int n, float acc) {
  const float r = g.res[b * g.res_bstride + (int64_t)m * g.ldo + n];
  g.out[b * g.out_bstride + (int64_t)m * g.ldo + n] = r + acc;
}

// j = output column in [0, f)
template <typename T>
__device__ __forceinline__ void epi_swiglu(const pt_gemm_args& g, int b, int m, int j, float gate, float up) {
  elem<T>::st((T*)g.olp + b * g.olp_bstride + (int64_t)m * (g.N >> 1) + j, silu_f(gate) * up);
}

// q or k section.  n0 = physical column of the low half (n0 % hd < hd/2); partner = n0 + hd/2.
template <typename T>
__device__ __forceinline__ void epi_rope_pair(const pt_gemm_args& g, int b, int m, int n0, float lo, float hi) {
  const int hq = g.H * g.hd, half = g.hd >> 1;
  const pt_rowpos rp = gemm_row_pos(g, m);
  const int seq = rp.seq, pos = rp.pos;
  const bool is_q = n0 < hq;
  const int c = is_q ? n0 : n0 - hq;
  const int head = c / g.hd, j = c - head * g.hd;
  const float2 cs = ((const float2*)g.rope)[(int64_t)pos * half + j];
  const float rlo = lo * cs.x - hi * cs.y;
  const float rhi = hi * cs.x + lo * cs.y;
  if (is_q) {
    T* q = (T*)g.olp + b * g.olp_bstride + (int64_t)m * hq + n0;
    elem<T>::st(q, rlo);
    elem<T>::st(q + half, rhi);
  } else {
    const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
    T* k = (T*)g.kc + hidx * g.kv_head_elems + (int64_t)pos * g.hd + j;
    elem<T>::st(k, rlo);
    elem<T>::st(k + half, rhi);
  }
}

// v section.  n = physical column (>= hq + hk).
template <typename T>
__device__ __forceinline__ void epi_v(const pt_gemm_args& g, int b, int m, int n, float acc) {
  const int c = n - (g.H + g.Hkv) * g.hd;
  const int head = c / g.hd, j = c - head * g.hd;
  const pt_rowpos rp = gemm_row_pos(g, m);
  const int seq = rp.seq, pos = rp.pos;
  const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
  elem<T>::st((T*)g.vc + hidx * ((int64_t)g.hd * g.s_pad) + (int64_t)j * g.s_pad + pos, acc);
}

#endif  // PT_EPILOGUE_H_

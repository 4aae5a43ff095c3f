// Causal flash-style prefill attention on the gfx950 matrix cores (bf16 operands, fp32 softmax).
//
// One wavefront owns 32 query rows of one (track, sequence, head) and walks the keys in blocks of
// 32.  Everything is computed transposed so that no operand ever needs a transpose:
//
//   S^T [32 keys x 32 queries] = K_blk [32 x hd] . Q^T          (A = K rows, B = Q rows; both hd-contiguous)
//   O^T [hd x 32 queries]     += V^T_blk [hd x 32 keys] . P^T   (A = rows of the V^T cache, key-contiguous;
//                                                                B = P^T straight from the S^T registers)
//
// In the S^T accumulator a lane holds one query column (lane % 32) and 16 keys, which is exactly the
// B-operand layout of the second product, so the probabilities never leave the lane's registers.  The
// softmax statistics (running max and sum) are per query = per lane; the two half-waves that share a
// query combine their maxima with one cross-lane exchange per key block.  The accumulator of O^T also
// has the query in the lane, so the online-softmax rescale is a per-lane multiply.
//
// Key order inside a block: MFMA row r of S^T is loaded from key pi(r) (r with bits 2 and 3 swapped),
// which makes the 8 probabilities a half-wave feeds to one PV MFMA eight consecutive keys - one 16-byte
// read of a V^T row.
#include "pt_device.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

union pk8 {
  bf16x8_t v;
  uint32_t u[4];
};

template <int HD>
__global__ void __launch_bounds__(256) attn_prefill_mfma_kernel(const pt_attn_args a) {
  constexpr int KS = HD / 16;   // MFMAs per S^T block
  constexpr int HB = HD / 32;   // 32-row blocks of O^T
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int qblocks = gridDim.x;
  const int qb = qblocks - 1 - (int)blockIdx.x;   // heavy (late) query blocks first
  const int q0 = qb * 128 + wave * 32;
  if (q0 >= a.S) return;
  const int head = blockIdx.y;
  const int t = blockIdx.z / a.B, seq = blockIdx.z - t * a.B;
  const int kvh = head / (a.H / a.Hkv);
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const bf16_t* K = (const bf16_t*)a.kc + hidx * a.kv_head_elems;
  const bf16_t* Vt = (const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad);
  const int64_t row = (int64_t)seq * a.S + q0 + l32;
  const int64_t qoff = t * a.q_bstride + row * (a.H * HD) + head * HD;
  const bf16_t* qrow = (const bf16_t*)a.q + qoff;

  bf16x8_t qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = *(const bf16x8_t*)(qrow + kk * 16 + half * 8);

  const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);   // pi(l32)
  const bf16_t* kptr = K + (int64_t)krow * HD + half * 8;
  const bf16_t* vptr = Vt + (int64_t)l32 * a.s_pad + 8 * half;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);

  f32x16_t oacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[hb][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int nkb = q0 / 32 + 1;
  for (int kb = 0; kb < nkb; ++kb) {
    f32x16_t s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
    const bf16_t* kp = kptr + (int64_t)kb * 32 * HD;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const bf16x8_t kf = *(const bf16x8_t*)(kp + kk * 16);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
    }
    // register v of this lane: key kb*32 + 16*(v/8) + 8*half + v%8, query q0 + l32
    float mx = -INFINITY;
    if (kb == nkb - 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key_in = 16 * (v >> 3) + 8 * half + (v & 7);
        s[v] = key_in > l32 ? -INFINITY : s[v] * scale_log2;
        mx = fmaxf(mx, s[v]);
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        s[v] *= scale_log2;
        mx = fmaxf(mx, s[v]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s[v] = __builtin_amdgcn_exp2f(s[v] - m_new);
      psum += s[v];
    }
    l_run = l_run * corr + psum;
    m_run = m_new;
    if (__any(corr != 1.0f)) {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[hb][v] *= corr;
    }
    pk8 pf[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) pf[u].u[i] = pack_bf16x2(s[8 * u + 2 * i], s[8 * u + 2 * i + 1]);
    const bf16_t* vp = vptr + kb * 32;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8_t vf = *(const bf16x8_t*)(vp + (int64_t)hb * 32 * a.s_pad + 16 * u);
        oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u].v, oacc[hb], 0, 0, 0);
      }
  }
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l;
  bf16_t* orow = (bf16_t*)a.o + qoff;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      uint2 pk;
      pk.x = pack_bf16x2(oacc[hb][vg * 4 + 0] * inv, oacc[hb][vg * 4 + 1] * inv);
      pk.y = pack_bf16x2(oacc[hb][vg * 4 + 2] * inv, oacc[hb][vg * 4 + 3] * inv);
      *(uint2*)(orow + hb * 32 + 8 * vg + 4 * half) = pk;
    }
}

int pt_launch_attn_prefill_mfma(const pt_attn_args& a, hipStream_t s) {
  if (a.dtype != PT_BF16 || a.pos0 != 0) return 0;
  if (a.hd != 64 && a.hd != 128) return 0;
  if (a.S < 32 || a.S % 32) return 0;
  if ((a.q_bstride & 7) || (((uintptr_t)a.q | (uintptr_t)a.o | (uintptr_t)a.kc | (uintptr_t)a.vc) & 15)) return 0;
  const int64_t z = (int64_t)a.n_tracks * a.B;
  if (z > 65535 || a.H > 65535) return 0;
  dim3 grid((unsigned)((a.S + 127) / 128), (unsigned)a.H, (unsigned)z);
  if (a.hd == 64)
    hipLaunchKernelGGL(attn_prefill_mfma_kernel<64>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(attn_prefill_mfma_kernel<128>, grid, dim3(256), 0, s, a);
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

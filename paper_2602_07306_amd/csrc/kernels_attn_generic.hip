// Shape-generic causal attention over the KV cache (prefill and decode), one wavefront per
// (query row, head): online softmax over chunks of 64 keys, fp32 arithmetic on the vector ALU.
// Serves the fp32 configuration and the shapes the tuned attention kernels do not cover.
#include "pt_device.h"

template <typename T>
__global__ void __launch_bounds__(64) attn_generic_kernel(pt_attn_args a) {
  __shared__ float qs[256];
  const int lane = threadIdx.x;
  const int m = blockIdx.x, head = blockIdx.y, t = blockIdx.z;
  const int hd = a.hd;
  int seq, pos;
  if (a.row_map) {   // ragged batch: decode rows are indexed by sequence, prefill rows by packed row
    const int2 e = a.row_map[m];
    seq = e.x;
    pos = e.y;
  } else {
    seq = m / a.S;
    pos = a.pos0 + (m - seq * a.S);
  }
  const int nkeys = pos + 1;
  const int kvh = head / (a.H / a.Hkv);
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const T* K = (const T*)a.kc + hidx * a.kv_head_elems;
  const T* Vt = (const T*)a.vc + hidx * ((int64_t)hd * a.s_pad);
  const int64_t qoff = t * a.q_bstride + (int64_t)m * a.H * hd + head * hd;
  const T* q = (const T*)a.q + qoff;
  for (int e = lane; e < hd; e += 64) qs[e] = elem<T>::ld(q + e);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float mrun = -INFINITY, lsum = 0.f;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int base = 0; base < nkeys; base += 64) {
    const int key = base + lane;
    float s = -INFINITY;
    if (key < nkeys) {
      const T* kr = K + (int64_t)key * hd;
      float dot = 0.f;
      for (int e = 0; e < hd; ++e) dot = fmaf(qs[e], elem<T>::ld(kr + e), dot);
      s = dot * scale;
    }
    const float mnew = fmaxf(mrun, wave_max(s));
    const float p = key < nkeys ? expf(s - mnew) : 0.f;
    const float corr = expf(mrun - mnew);   // 0 on the first chunk
    lsum = lsum * corr + wave_sum(p);
    mrun = mnew;
    const int nk = min(64, nkeys - base);
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] *= corr;
    for (int kk = 0; kk < nk; ++kk) {
      const float pk = __shfl(p, kk, 64);   // executed by the whole wavefront
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e = lane + 64 * i;
        if (e < hd) acc[i] = fmaf(pk, elem<T>::ld(Vt + (int64_t)e * a.s_pad + base + kk), acc[i]);
      }
    }
  }
  T* o = (T*)a.o + qoff;
  const float inv = 1.0f / lsum;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int e = lane + 64 * i;
    if (e < hd) elem<T>::st(o + e, acc[i] * inv);
  }
}

int pt_launch_attn_generic(const pt_attn_args& a, hipStream_t s) {
  const int64_t rows = a.seq_info ? a.rows : (int64_t)a.B * a.S;
  if (rows <= 0) return PT_OK;
  if (a.hd > 256) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "head_dim > 256");
  dim3 grid((unsigned)rows, (unsigned)a.H, (unsigned)a.n_tracks);
  if (a.dtype == PT_F32)
    hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(64), 0, s, a);
  else
    hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(64), 0, s, a);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// Shape-generic GEMM with the fused epilogues: any M, N, K (N even), fp32 or bf16 operands, fp32
// accumulation on the vector ALU.  It serves the fp32 configuration and every shape the MFMA
// family does not cover; it is written for clarity, not speed.
#include "pt_epilogue.h"

#define GG_BK 32

__device__ __forceinline__ void pair_columns(const pt_gemm_args& g, int p, int* n0, int* n1) {
  if (g.epi == EPI_SWIGLU) {
    *n0 = swiglu_gate_row(p);
    *n1 = *n0 + 32;
  } else if (g.epi == EPI_QKV) {
    const int half = g.hd >> 1, rot_pairs = (g.H + g.Hkv) * half;
    if (p < rot_pairs) {
      const int head = p / half, j = p - head * half;
      *n0 = head * g.hd + j;
      *n1 = *n0 + half;
    } else {
      *n0 = (g.H + g.Hkv) * g.hd + 2 * (p - rot_pairs);
      *n1 = *n0 + 1;
    }
  } else {
    *n0 = 2 * p;
    *n1 = 2 * p + 1;
  }
}

template <typename T>
__global__ void __launch_bounds__(256) gemm_generic_kernel(pt_gemm_args g) {
  __shared__ float As[16][GG_BK + 1];
  __shared__ float W0s[16][GG_BK + 1];
  __shared__ float W1s[16][GG_BK + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int b = blockIdx.z;
  const int m0 = blockIdx.y * 16, p0 = blockIdx.x * 16;
  const int npairs = g.N >> 1;
  const T* A = (const T*)g.A + b * g.a_bstride;
  const T* W = (const T*)g.W + b * g.w_bstride;
  if (g.blk_group) {   // grouped GEMM: weight matrix by 64-row block; blocks without rows are skipped
    const int group = g.blk_group[b * g.grp_bstride + (m0 >> 6)];
    if (group < 0) return;
    W += group * g.w_gstride;
  }
  // row of A behind tile row ty (a gather when a_rows is given)
  const int64_t arow = m0 + ty < g.M ? (g.a_rows ? g.a_rows[b * g.a_rows_bstride + m0 + ty] : m0 + ty) : 0;

  // the W rows this block needs, one pair per tile row
  int ln0 = 0, ln1 = 0;
  {
    const int p = p0 + ty;
    if (p < npairs) pair_columns(g, p, &ln0, &ln1);
  }
  float acc0 = 0.f, acc1 = 0.f;
  for (int k0 = 0; k0 < g.K; k0 += GG_BK) {
    for (int e = tx; e < GG_BK; e += 16) {
      const int k = k0 + e;
      const bool kin = k < g.K;
      As[ty][e] = (kin && m0 + ty < g.M) ? elem<T>::ld(A + arow * g.lda + k) : 0.f;
      const bool pin = kin && (p0 + ty) < npairs;
      W0s[ty][e] = pin ? elem<T>::ld(W + (int64_t)ln0 * g.ldb + k) : 0.f;
      W1s[ty][e] = pin ? elem<T>::ld(W + (int64_t)ln1 * g.ldb + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < GG_BK; ++e) {
      const float a = As[ty][e];
      acc0 = fmaf(a, W0s[tx][e], acc0);
      acc1 = fmaf(a, W1s[tx][e], acc1);
    }
    __syncthreads();
  }
  const int m = m0 + ty, p = p0 + tx;
  if (m >= g.M || p >= npairs) return;
  int n0, n1;
  pair_columns(g, p, &n0, &n1);
  switch (g.epi) {
    case EPI_STORE_F32:
      epi_store_f32<T>(g, b, m, n0, acc0);
      epi_store_f32<T>(g, b, m, n1, acc1);
      break;
    case EPI_RESIDUAL:
      epi_residual<T>(g, b, m, n0, acc0);
      epi_residual<T>(g, b, m, n1, acc1);
      break;
    case EPI_SWIGLU:
      epi_swiglu<T>(g, b, m, p, acc0, acc1);
      break;
    case EPI_QKV:
      if (n0 < (g.H + g.Hkv) * g.hd) {
        epi_rope_pair<T>(g, b, m, n0, acc0, acc1);
      } else {
        epi_v<T>(g, b, m, n0, acc0);
        epi_v<T>(g, b, m, n1, acc1);
      }
      break;
  }
}

int pt_launch_gemm_generic(const pt_gemm_args& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return PT_OK;
  if (g.N & 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "generic GEMM needs an even N");
  dim3 grid((unsigned)((g.N / 2 + 15) / 16), (unsigned)((g.M + 15) / 16), (unsigned)g.batch);
  if (grid.y > 65535u) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "generic GEMM: M too large");
  if (g.dtype == PT_F32)
    hipLaunchKernelGGL(gemm_generic_kernel<float>, grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_generic_kernel<bf16_t>, grid, dim3(256), 0, s, g);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

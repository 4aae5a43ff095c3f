// Bandwidth-bound kernels of the PT forward: embedding gather, RMSNorm, the track merge of
// Algorithm 1 (Section 2.2), argmax, the rotary table, and small copies.
#include "pt_device.h"

// ------------------------------------------------------------------------------------------
// Embedding: h[row, :] = E[token[row], :] as fp32.  An id outside [0, vocab) reads the nearest table row (so
// that no access leaves the table) and sets bit 0 of the device status word, which pt_sync_status reports.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) embed_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok,
                                                    int64_t rows, int32_t d, int32_t vocab, float* __restrict__ h,
                                                    int32_t* __restrict__ flag) {
  const int64_t row = blockIdx.x;
  if (row >= rows) return;
  int32_t id = tok[row];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0 && flag) atomicOr(flag, 1);
    id = id < 0 ? 0 : vocab - 1;
  }
  const T* src = E + (int64_t)id * d;
  float* dst = h + row * d;
  for (int c = threadIdx.x; c < d; c += 256) dst[c] = elem<T>::ld(src + c);
}

int pt_launch_embed(const void* embed, int32_t dtype, const int32_t* tokens, int64_t rows, int32_t d,
                    int32_t vocab, float* h, int32_t* flag, hipStream_t s) {
  if (rows <= 0) return PT_OK;
  if (dtype == PT_F32)
    hipLaunchKernelGGL(embed_kernel<float>, dim3((unsigned)rows), dim3(256), 0, s, (const float*)embed, tokens, rows, d, vocab, h, flag);
  else
    hipLaunchKernelGGL(embed_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, s, (const bf16_t*)embed, tokens, rows, d, vocab, h, flag);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------
// Ragged batches (sequences of different lengths in one prefill).  Inside the library the rows of a ragged
// prefill are packed sequence after sequence, each padded to a multiple of 64 rows; padding rows carry the zero
// vector as their input and run through the layers like appended tokens, which the causal mask keeps away from
// every real position.  seq_info[b] = (first packed row, padded length, length, first token of the packed input).
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) embed_ragged_kernel(const T* __restrict__ E, const int32_t* __restrict__ tok,
                                                           const int2* __restrict__ row_map, const int4* __restrict__ seq_info,
                                                           int64_t rows, int32_t d, int32_t vocab, float* __restrict__ h,
                                                           int32_t* __restrict__ flag) {
  const int64_t row = blockIdx.x;
  if (row >= rows) return;
  const int2 rp = row_map[row];
  const int4 si = seq_info[rp.x];
  float* dst = h + row * d;
  if (rp.y >= si.z) {
    for (int c = threadIdx.x; c < d; c += 256) dst[c] = 0.f;
    return;
  }
  int32_t id = tok[si.w + rp.y];
  if (id < 0 || id >= vocab) {
    if (threadIdx.x == 0 && flag) atomicOr(flag, 1);
    id = id < 0 ? 0 : vocab - 1;
  }
  const T* src = E + (int64_t)id * d;
  for (int c = threadIdx.x; c < d; c += 256) dst[c] = elem<T>::ld(src + c);
}

int pt_launch_embed_ragged(const void* embed, int32_t dtype, const int32_t* tokens, const int2* row_map,
                           const int4* seq_info, int64_t rows, int32_t d, int32_t vocab, float* h, int32_t* flag,
                           hipStream_t s) {
  if (rows <= 0) return PT_OK;
  if (dtype == PT_F32)
    hipLaunchKernelGGL(embed_ragged_kernel<float>, dim3((unsigned)rows), dim3(256), 0, s, (const float*)embed, tokens, row_map, seq_info, rows, d, vocab, h, flag);
  else
    hipLaunchKernelGGL(embed_ragged_kernel<bf16_t>, dim3((unsigned)rows), dim3(256), 0, s, (const bf16_t*)embed, tokens, row_map, seq_info, rows, d, vocab, h, flag);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

__global__ void __launch_bounds__(256) scatter_rows_kernel(const float* __restrict__ src, int64_t src_bstride,
                                                           const int2* __restrict__ row_map, const int4* __restrict__ seq_info,
                                                           int32_t d, float* __restrict__ dst, int64_t dst_bstride) {
  const int64_t row = blockIdx.x;
  const int b = blockIdx.y;
  const int2 rp = row_map[row];
  const int4 si = seq_info[rp.x];
  float4* o = (float4*)(dst + b * dst_bstride + row * d);
  if (rp.y >= si.z) {
    for (int c = threadIdx.x; c < (d >> 2); c += 256) o[c] = make_float4(0.f, 0.f, 0.f, 0.f);
    return;
  }
  const float4* in = (const float4*)(src + b * src_bstride + (int64_t)(si.w + rp.y) * d);
  for (int c = threadIdx.x; c < (d >> 2); c += 256) o[c] = in[c];
}

int pt_launch_scatter_rows(const float* src, int64_t src_bstride, const int2* row_map, const int4* seq_info,
                           int64_t rows, int32_t d, int32_t batch, float* dst, int64_t dst_bstride, hipStream_t s) {
  if (rows <= 0 || batch <= 0) return PT_OK;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3((unsigned)rows, (unsigned)batch), dim3(256), 0, s, src, src_bstride, row_map,
                     seq_info, d, dst, dst_bstride);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

__global__ void __launch_bounds__(256) gather_rows_kernel(const float* __restrict__ src, const int32_t* __restrict__ idx,
                                                          int32_t d, float* __restrict__ dst) {
  const int64_t i = blockIdx.x;
  const float4* in = (const float4*)(src + (int64_t)idx[i] * d);
  float4* o = (float4*)(dst + i * d);
  for (int c = threadIdx.x; c < (d >> 2); c += 256) o[c] = in[c];
}

int pt_launch_gather_rows(const float* src, const int32_t* idx, int64_t n, int32_t d, float* dst, hipStream_t s) {
  if (n <= 0) return PT_OK;
  hipLaunchKernelGGL(gather_rows_kernel, dim3((unsigned)n), dim3(256), 0, s, src, idx, d, dst);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// One workgroup per sequence: its packed rows get (sequence, position), its real tokens their packed row.
__global__ void __launch_bounds__(256) ragged_maps_kernel(const int4* __restrict__ seq_info, int2* __restrict__ row_map,
                                                          int32_t* __restrict__ valid, int32_t* __restrict__ last) {
  const int b = blockIdx.x;
  const int4 si = seq_info[b];
  for (int p = threadIdx.x; p < si.y; p += 256) row_map[si.x + p] = make_int2(b, p);
  for (int p = threadIdx.x; p < si.z; p += 256) valid[si.w + p] = si.x + p;
  if (threadIdx.x == 0) last[b] = si.x + si.z - 1;
}

int pt_launch_ragged_maps(const int4* seq_info, int32_t B, int64_t rows, int2* row_map, int32_t* valid, int32_t* last,
                          hipStream_t s) {
  (void)rows;
  if (B <= 0) return PT_OK;
  hipLaunchKernelGGL(ragged_maps_kernel, dim3((unsigned)B), dim3(256), 0, s, seq_info, row_map, valid, last);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

__global__ void __launch_bounds__(256) decode_rowmap_kernel(const int4* __restrict__ seq_info, int32_t B, int2* __restrict__ row_map) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < B) row_map[b] = make_int2(b, seq_info[b].z);
}

__global__ void __launch_bounds__(256) advance_lens_kernel(int4* __restrict__ seq_info, int32_t B) {
  const int b = blockIdx.x * 256 + threadIdx.x;
  if (b < B) seq_info[b].z += 1;
}

int pt_launch_decode_rowmap(int4* seq_info, int32_t B, int2* row_map, hipStream_t s) {
  if (B <= 0) return PT_OK;
  hipLaunchKernelGGL(decode_rowmap_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, s, seq_info, B, row_map);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

int pt_launch_advance_lens(int4* seq_info, int32_t B, hipStream_t s) {
  if (B <= 0) return PT_OK;
  hipLaunchKernelGGL(advance_lens_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, s, seq_info, B);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------
// RMSNorm: out = h * g / sqrt(mean(h^2) + eps); fp32 statistics; one wavefront per row.
// Row r of track b reads h + b*h_bstride + row_index(r)*d with row_index(r) = r*row_step + row_off.
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void store4(float* p, float a, float b, float c, float d) {
  *(float4*)p = make_float4(a, b, c, d);
}
__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
  uint2 v;
  v.x = pack_bf16x2(a, b);
  v.y = pack_bf16x2(c, d);
  *(uint2*)p = v;
}

template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_kernel(const float* __restrict__ h, int64_t h_bstride,
                                                      const float* __restrict__ gains, int64_t g_bstride,
                                                      T* __restrict__ out, int64_t out_bstride, int64_t rows,
                                                      int64_t row_step, int64_t row_off,
                                                      const int32_t* __restrict__ row_idx, int32_t d, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t r = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int b = blockIdx.y;
  if (r >= rows) return;
  const int64_t sr = row_idx ? (int64_t)row_idx[r] : r * row_step + row_off;
  const float4* src = (const float4*)(h + b * h_bstride + sr * d);
  const float4* g = (const float4*)(gains + b * g_bstride);
  const int n4 = d >> 2;
  float ss = 0.f;
  for (int i = lane; i < n4; i += 64) {
    float4 v = src[i];
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T* dst = out + b * out_bstride + r * d;
  for (int i = lane; i < n4; i += 64) {
    float4 v = src[i];
    float4 w = g[i];
    store4(dst + 4 * i, v.x * inv * w.x, v.y * inv * w.y, v.z * inv * w.z, v.w * inv * w.w);
  }
}

// Few rows (decode): one workgroup per row, so that a long row is not read by a single wavefront.
template <typename T>
__global__ void __launch_bounds__(256) rmsnorm_row_kernel(const float* __restrict__ h, int64_t h_bstride,
                                                          const float* __restrict__ gains, int64_t g_bstride,
                                                          T* __restrict__ out, int64_t out_bstride, int64_t rows,
                                                          int64_t row_step, int64_t row_off,
                                                          const int32_t* __restrict__ row_idx, int32_t d, float eps) {
  __shared__ float s_part[4];
  const int64_t r = blockIdx.x;
  const int b = blockIdx.y;
  const int64_t sr = row_idx ? (int64_t)row_idx[r] : r * row_step + row_off;
  const float4* src = (const float4*)(h + b * h_bstride + sr * d);
  const float4* g = (const float4*)(gains + b * g_bstride);
  const int n4 = d >> 2;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 v = src[i];
    ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  T* dst = out + b * out_bstride + r * d;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 v = src[i];
    float4 w = g[i];
    store4(dst + 4 * i, v.x * inv * w.x, v.y * inv * w.y, v.z * inv * w.z, v.w * inv * w.w);
  }
}

// Decode residual GEMMs with K split over workgroups leave `slices` partial products; this kernel adds them
// to the residual stream, stores the stream and (when out is given) its RMSNorm for the next GEMM.
// One workgroup per row; a thread keeps its <= 32 elements in registers between the two passes.
__global__ void __launch_bounds__(256) resnorm_kernel(const float* __restrict__ part, int32_t slices,
                                                      const float* res, int64_t res_bstride, float* h,
                                                      int64_t h_bstride, const float* __restrict__ gains,
                                                      int64_t g_bstride, bf16_t* __restrict__ out,
                                                      int64_t out_bstride, int32_t batch, int64_t rows, int32_t d,
                                                      float eps) {
  __shared__ float s_part[4];
  const int64_t r = blockIdx.x;
  const int b = blockIdx.y;
  const int n4 = d >> 2;
  const float4* rsrc = (const float4*)(res + b * res_bstride + r * d);
  float4* hdst = (float4*)(h + b * h_bstride + r * d);
  const int64_t slice_stride4 = ((int64_t)batch * rows * d) >> 2;
  const float4* p0 = (const float4*)part + (((int64_t)b * rows + r) * d >> 2);
  float4 x[8];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int i = threadIdx.x + c * 256;
    if (i < n4) {
      float4 acc = p0[i];
      for (int q = 1; q < slices; ++q) {
        const float4 v = p0[q * slice_stride4 + i];
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
      const float4 rv = rsrc[i];
      acc.x += rv.x; acc.y += rv.y; acc.z += rv.z; acc.w += rv.w;
      hdst[i] = acc;
      x[c] = acc;
      ss += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
    }
  }
  if (!out) return;
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  const float4* g = (const float4*)(gains + b * g_bstride);
  bf16_t* dst = out + b * out_bstride + r * d;
#pragma unroll
  for (int c = 0; c < 8; ++c) {
    const int i = threadIdx.x + c * 256;
    if (i < n4) {
      const float4 w = g[i];
      store4(dst + 4 * i, x[c].x * inv * w.x, x[c].y * inv * w.y, x[c].z * inv * w.z, x[c].w * inv * w.w);
    }
  }
}

int pt_launch_resnorm(const float* part, int32_t slices, const float* res, int64_t res_bstride, float* h,
                      int64_t h_bstride, const float* gains, int64_t g_bstride, void* out, int64_t out_bstride,
                      int32_t batch, int64_t rows, int32_t d, float eps, hipStream_t s) {
  if (rows <= 0 || batch <= 0) return PT_OK;
  if (d > 8192 || (d & 3) || slices < 1) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "resnorm: d = %d, slices = %d not covered", d, slices);
  hipLaunchKernelGGL(resnorm_kernel, dim3((unsigned)rows, (unsigned)batch), dim3(256), 0, s, part, slices, res,
                     res_bstride, h, h_bstride, gains, g_bstride, (bf16_t*)out, out_bstride, batch, rows, d, eps);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

static int launch_rmsnorm(const float* h, int64_t h_bstride, const float* gains, int64_t g_bstride, void* out,
                          int64_t out_bstride, int32_t dtype, int32_t batch, int64_t rows, int64_t row_step,
                          int64_t row_off, const int32_t* row_idx, int32_t d, float eps, hipStream_t s) {
  if (rows <= 0 || batch <= 0) return PT_OK;
  if (rows * batch <= 2048 && d >= 1024) {
    dim3 grid((unsigned)rows, (unsigned)batch);
    if (dtype == PT_F32)
      hipLaunchKernelGGL(rmsnorm_row_kernel<float>, grid, dim3(256), 0, s, h, h_bstride, gains, g_bstride, (float*)out,
                         out_bstride, rows, row_step, row_off, row_idx, d, eps);
    else
      hipLaunchKernelGGL(rmsnorm_row_kernel<bf16_t>, grid, dim3(256), 0, s, h, h_bstride, gains, g_bstride, (bf16_t*)out,
                         out_bstride, rows, row_step, row_off, row_idx, d, eps);
    PT_HIP_CHECK(hipGetLastError());
    return PT_OK;
  }
  dim3 grid((unsigned)((rows + 3) / 4), (unsigned)batch);
  if (dtype == PT_F32)
    hipLaunchKernelGGL(rmsnorm_kernel<float>, grid, dim3(256), 0, s, h, h_bstride, gains, g_bstride, (float*)out,
                       out_bstride, rows, row_step, row_off, row_idx, d, eps);
  else
    hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, grid, dim3(256), 0, s, h, h_bstride, gains, g_bstride, (bf16_t*)out,
                       out_bstride, rows, row_step, row_off, row_idx, d, eps);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

int pt_launch_rmsnorm(const float* h, int64_t h_bstride, const float* gains, int64_t g_bstride, void* out,
                      int64_t out_bstride, int32_t dtype, int32_t batch, int64_t rows, int32_t d, float eps,
                      hipStream_t s) {
  return launch_rmsnorm(h, h_bstride, gains, g_bstride, out, out_bstride, dtype, batch, rows, 1, 0, nullptr, d, eps, s);
}

int pt_launch_rmsnorm_rows(const float* h, const float* gain, void* out, int32_t dtype, int64_t rows,
                           int64_t row_step, int64_t row_off, const int32_t* row_idx, int32_t d, float eps, hipStream_t s) {
  return launch_rmsnorm(h, 0, gain, 0, out, 0, dtype, 1, rows, row_step, row_off, row_idx, d, eps, s);
}

// ------------------------------------------------------------------------------------------
// Track merge (the all-reduce of Algorithm 1 on one device):
//   out = scale * (t_0 + t_1 + ... + t_{n-1}), fp32 accumulation in track order.
// Each thread owns 8 consecutive elements per step: every track is read exactly once with 16-byte
// (bf16) or 2 x 16-byte (fp32) loads and the result is written exactly once.
// ------------------------------------------------------------------------------------------
struct merge_ptrs {
  const void* t[16];
};

template <typename T>
__global__ void __launch_bounds__(256) merge_kernel(merge_ptrs p, int n, int64_t chunks, float scale,
                                                    T* __restrict__ out, float* __restrict__ tap);

template <>
__global__ void __launch_bounds__(256) merge_kernel<float>(merge_ptrs p, int n, int64_t chunks, float scale,
                                                           float* __restrict__ out, float* __restrict__ tap) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += stride) {
    float4 a0 = ((const float4*)p.t[0])[2 * c], a1 = ((const float4*)p.t[0])[2 * c + 1];
    for (int i = 1; i < n; ++i) {
      const float4 b0 = ((const float4*)p.t[i])[2 * c], b1 = ((const float4*)p.t[i])[2 * c + 1];
      a0.x += b0.x; a0.y += b0.y; a0.z += b0.z; a0.w += b0.w;
      a1.x += b1.x; a1.y += b1.y; a1.z += b1.z; a1.w += b1.w;
    }
    a0.x *= scale; a0.y *= scale; a0.z *= scale; a0.w *= scale;
    a1.x *= scale; a1.y *= scale; a1.z *= scale; a1.w *= scale;
    ((float4*)out)[2 * c] = a0;
    ((float4*)out)[2 * c + 1] = a1;
    if (tap) {
      ((float4*)tap)[2 * c] = a0;
      ((float4*)tap)[2 * c + 1] = a1;
    }
  }
}

template <>
__global__ void __launch_bounds__(256) merge_kernel<bf16_t>(merge_ptrs p, int n, int64_t chunks, float scale,
                                                            bf16_t* __restrict__ out, float* __restrict__ tap) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x; c < chunks; c += stride) {
    float acc[8];
    {
      const uint4 v = ((const uint4*)p.t[0])[c];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] = __uint_as_float(w[k] << 16);
        acc[2 * k + 1] = __uint_as_float(w[k] & 0xffff0000u);
      }
    }
    for (int i = 1; i < n; ++i) {
      const uint4 v = ((const uint4*)p.t[i])[c];
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[2 * k] += __uint_as_float(w[k] << 16);
        acc[2 * k + 1] += __uint_as_float(w[k] & 0xffff0000u);
      }
    }
    uint4 o;
    o.x = pack_bf16x2(acc[0] * scale, acc[1] * scale);
    o.y = pack_bf16x2(acc[2] * scale, acc[3] * scale);
    o.z = pack_bf16x2(acc[4] * scale, acc[5] * scale);
    o.w = pack_bf16x2(acc[6] * scale, acc[7] * scale);
    ((uint4*)out)[c] = o;
  }
}

int pt_launch_merge(const void* const* tracks, int32_t n, int64_t elems, int32_t dtype, float scale, void* out,
                    float* tap, hipStream_t s) {
  if (elems <= 0) return PT_OK;
  merge_ptrs p;
  for (int i = 0; i < 16; ++i) p.t[i] = i < n ? tracks[i] : nullptr;
  const int64_t chunks = elems / 8;
  int64_t blocks = (chunks + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (dtype == PT_F32)
    hipLaunchKernelGGL(merge_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, p, n, chunks, scale, (float*)out, tap);
  else
    hipLaunchKernelGGL(merge_kernel<bf16_t>, dim3((unsigned)blocks), dim3(256), 0, s, p, n, chunks, scale, (bf16_t*)out, tap);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) copy_f32_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t n) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

int pt_launch_copy_f32(const float* src, float* dst, int64_t elems, hipStream_t s) {
  if (elems <= 0) return PT_OK;
  int64_t blocks = (elems + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(copy_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, src, dst, elems);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

__global__ void __launch_bounds__(256) fill_f32_kernel(float* __restrict__ dst, int64_t n, float v) {
  const int64_t stride = (int64_t)gridDim.x * 256;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = v;
}

// RMSNorm folded into the GEMMs around it: the residual GEMM leaves `parts` partial sums of squares per row; this
// turns them into the row's factor 1 / sqrt(mean + eps), summed in part order.
__global__ void __launch_bounds__(256) row_inv_rms_kernel(const float* __restrict__ ss, int32_t parts, int64_t rows,
                                                          float inv_d, float eps, float* __restrict__ out) {
  const int64_t r = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (r >= rows) return;
  const float* p = ss + r * parts;
  float acc = 0.f;
  for (int q = 0; q < parts; ++q) acc += p[q];
  out[r] = 1.0f / sqrtf(acc * inv_d + eps);
}

int pt_launch_row_inv_rms(const float* ss, int32_t parts, int64_t rows, int32_t d, float eps, float* out, hipStream_t s) {
  if (rows <= 0) return PT_OK;
  hipLaunchKernelGGL(row_inv_rms_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, s, ss, parts, rows,
                     1.0f / (float)d, eps, out);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

int pt_launch_fill_f32(float* dst, int64_t n, float v, hipStream_t s) {
  if (n <= 0) return PT_OK;
  int64_t blocks = (n + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(fill_f32_kernel, dim3((unsigned)blocks), dim3(256), 0, s, dst, n, v);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------
// Greedy token: argmax over the vocabulary, lowest id on ties.  One workgroup per row.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) argmax_kernel(const float* __restrict__ logits, int32_t vocab, int32_t* __restrict__ out) {
  __shared__ float sv[256];
  __shared__ int32_t si[256];
  const float* row = logits + (int64_t)blockIdx.x * vocab;
  float best = -INFINITY;
  int32_t bi = 0x7fffffff;
  // 16-byte loads, four in flight per thread (vocab is a multiple of 4 and rows are 16-byte aligned when the
  // logits buffer is; otherwise one element at a time)
  if ((vocab & 3) == 0 && ((uintptr_t)row & 15) == 0) {
    const int n4 = vocab >> 2;
    for (int i0 = threadIdx.x; i0 < n4; i0 += 4 * 256) {
      float4 v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i4 = i0 + u * 256;
        v[u] = i4 < n4 ? ((const float4*)row)[i4] : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (i0 + u * 256 >= n4) break;
        const int i = 4 * (i0 + u * 256);
        const float e[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (e[j] > best || (e[j] == best && i + j < bi)) { best = e[j]; bi = i + j; }
      }
    }
  } else {
    for (int i = threadIdx.x; i < vocab; i += 256) {
      const float v = row[i];
      if (v > best || (v == best && i < bi)) { best = v; bi = i; }
    }
  }
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bi;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if ((int)threadIdx.x < o) {
      const float v = sv[threadIdx.x + o];
      const int32_t i = si[threadIdx.x + o];
      if (v > sv[threadIdx.x] || (v == sv[threadIdx.x] && i < si[threadIdx.x])) { sv[threadIdx.x] = v; si[threadIdx.x] = i; }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) out[blockIdx.x] = si[0] == 0x7fffffff ? 0 : si[0];
}

int pt_launch_argmax(const float* logits, int32_t rows, int32_t vocab, int32_t* out, hipStream_t s) {
  if (rows <= 0) return PT_OK;
  hipLaunchKernelGGL(argmax_kernel, dim3((unsigned)rows), dim3(256), 0, s, logits, vocab, out);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------
// Rotary table: table[p][j] = (cos, sin)(p * theta^(-2j/hd)), angle evaluated in double.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) rope_table_kernel(float2* __restrict__ table, int32_t max_seq, int32_t half, double theta, int32_t hd) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= (int64_t)max_seq * half) return;
  const int p = (int)(i / half), j = (int)(i % half);
  const double inv_freq = pow(theta, -2.0 * (double)j / (double)hd);
  const double ang = (double)p * inv_freq;
  table[i] = make_float2((float)cos(ang), (float)sin(ang));
}

int pt_launch_rope_table(float* table, int32_t max_seq, int32_t hd, float theta, hipStream_t s) {
  const int half = hd / 2;
  const int64_t n = (int64_t)max_seq * half;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, (float2*)table, max_seq, half, (double)theta, hd);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// PT-MoE (Section 2.2 and the Conclusion of the paper: MoE sparsity inside every track): expert selection from
// the router logits, grouping of the (row, expert) assignments by expert for the grouped expert GEMMs, and the
// weighted combine of the expert outputs with the residual stream.
//
// Grouping.  Every row of a track chooses k of E experts; the track's rows * k assignments are laid out in
// `slots` so that the assignments of expert e are contiguous and start at a multiple of 256 (the largest GEMM
// tile height), in row order inside an expert.  The order is fixed by counting, not by atomics: per 256-row block
// the assignments per expert are counted (ballots), an exclusive scan over the blocks gives every block its first
// slot per expert, and the block's rows take consecutive slots in row order.  Slots between the end of an
// expert's assignments and the next multiple of 256 are padding: their row index is some valid row (the GEMMs
// compute them and nobody reads the result), and 64-slot blocks made of padding only are marked -1 so that GEMM
// tiles starting there return at once.
#include "pt_device.h"

#define MOE_ROWS 256   // rows per counting block

// ------------------------------------------------------------------------------------------------
// Top-k of E logits per row: k passes, each taking the largest logit not taken yet (strict >, so the lowest
// index wins exact ties), then the softmax over the k chosen logits.  One thread per (track, row).
// ------------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) moe_topk_kernel(pt_moe_args a) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)a.T * a.rows) return;
  const int t = (int)(idx / a.rows);
  const int64_t r = idx - (int64_t)t * a.rows;
  const float* lg = a.logits + idx * a.e_pad;
  int32_t* route = a.route + idx * a.k;
  float* gate = a.gate + idx * a.k;
  uint64_t taken = 0;
  float vmax = -INFINITY;
  bool bad = false;
  for (int j = 0; j < a.k; ++j) {
    int bi = -1;
    float best = -INFINITY;
    if (a.forced) {
      const int e = a.forced[t * a.obs_bstride + r * a.k + j];
      if (e >= 0 && e < a.E && !((taken >> e) & 1)) { bi = e; best = lg[e]; }
      else bad = true;
    } else {
      for (int e = 0; e < a.E; ++e) {
        const float v = lg[e];
        if (!((taken >> e) & 1) && v > best) { best = v; bi = e; }
      }
    }
    if (bi < 0) {   // nothing comparable left (NaN logits) or an invalid forced entry: lowest expert not taken
      bi = __ffsll((unsigned long long)~taken) - 1;
      best = lg[bi];
    }
    taken |= 1ull << bi;
    route[j] = bi;
    gate[j] = best;
    vmax = fmaxf(vmax, best);
    if (a.chosen_out) a.chosen_out[t * a.obs_bstride + r * a.k + j] = bi;
  }
  if (bad) atomicOr(a.flag, 2);
  float sum = 0.f;
  for (int j = 0; j < a.k; ++j) {
    const float w = expf(gate[j] - vmax);
    gate[j] = w;
    sum += w;
  }
  const float inv = 1.0f / sum;
  for (int j = 0; j < a.k; ++j) gate[j] *= inv;
}

// The k experts of a row packed one per byte, or 0xff..ff for rows past the end.
__device__ __forceinline__ uint64_t load_packed_route(const pt_moe_args& a, int t, int64_t r) {
  uint64_t packed = ~0ull;
  if (r < a.rows) {
    packed = 0;
    const int32_t* route = a.route + ((int64_t)t * a.rows + r) * a.k;
    for (int j = 0; j < a.k; ++j) packed |= (uint64_t)(uint8_t)route[j] << (8 * j);
  }
  return packed;
}
__device__ __forceinline__ int find_expert(uint64_t packed, int k, int e) {
  for (int j = 0; j < k; ++j)
    if ((int)((packed >> (8 * j)) & 0xff) == e) return j;
  return -1;
}

// Assignments per expert in each block of 256 rows; also presets the row-of-slot table for the padding slots.
__global__ void __launch_bounds__(MOE_ROWS) moe_count_kernel(pt_moe_args a, int nblk) {
  __shared__ int s_cnt[4][64];
  const int blk = blockIdx.x, t = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // padding slots read some valid row; spread them over the rows, since thousands of loads of one row would all
  // queue on one memory channel
  for (int64_t i = (int64_t)blk * MOE_ROWS + tid; i < a.slots; i += (int64_t)nblk * MOE_ROWS)
    a.perm[t * a.slots + i] = (int32_t)(i % a.rows);
  const uint64_t packed = load_packed_route(a, t, (int64_t)blk * MOE_ROWS + tid);
  for (int e = 0; e < a.E; ++e) {
    const uint64_t bal = __ballot(find_expert(packed, a.k, e) >= 0);
    if (lane == 0) s_cnt[wave][e] = __popcll(bal);
  }
  __syncthreads();
  if (tid < 64)
    a.cnt[((int64_t)t * (nblk + 2) + blk) * 64 + tid] = tid < a.E ? (s_cnt[0][tid] + s_cnt[1][tid]) + (s_cnt[2][tid] + s_cnt[3][tid]) : 0;
}

// Per track (one wavefront, lane = expert): exclusive scan of the block counts, totals, 256-aligned segment
// bases, and the expert of every 64-slot block.
__global__ void __launch_bounds__(64) moe_scan_kernel(pt_moe_args a, int nblk) {
  __shared__ int s_pad[64];
  const int t = blockIdx.x, e = threadIdx.x;
  int32_t* cnt = a.cnt + (int64_t)t * (nblk + 2) * 64;
  int running = 0;
  for (int blk = 0; blk < nblk; ++blk) {
    const int v = cnt[blk * 64 + e];
    cnt[blk * 64 + e] = running;
    running += v;
  }
  cnt[nblk * 64 + e] = running;
  s_pad[e] = (running + 255) / 256 * 256;
  __syncthreads();
  int base = 0;
  for (int i = 0; i < e; ++i) base += s_pad[i];
  cnt[(nblk + 1) * 64 + e] = base;
  int32_t* blk_e = a.blk + t * (a.slots / 64);
  for (int64_t i = e; i < a.slots / 64; i += 64) blk_e[i] = -1;
  __syncthreads();
  const int used = (running + 63) / 64;
  for (int i = 0; i < used; ++i) blk_e[base / 64 + i] = e;
}

// Slot of every assignment (row order inside an expert) and row of every slot.
__global__ void __launch_bounds__(MOE_ROWS) moe_place_kernel(pt_moe_args a, int nblk) {
  __shared__ int s_cnt[4][64];
  const int blk = blockIdx.x, t = blockIdx.y, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int64_t r = (int64_t)blk * MOE_ROWS + tid;
  const uint64_t packed = load_packed_route(a, t, r);
  for (int e = 0; e < a.E; ++e) {
    const uint64_t bal = __ballot(find_expert(packed, a.k, e) >= 0);
    if (lane == 0) s_cnt[wave][e] = __popcll(bal);
  }
  __syncthreads();
  const int32_t* cnt = a.cnt + (int64_t)t * (nblk + 2) * 64;
  const uint64_t below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  for (int e = 0; e < a.E; ++e) {
    const int j = find_expert(packed, a.k, e);
    const uint64_t bal = __ballot(j >= 0);
    if (j >= 0) {
      int before = __popcll(bal & below);
      for (int w = 0; w < wave; ++w) before += s_cnt[w][e];
      const int slot = cnt[(nblk + 1) * 64 + e] + cnt[blk * 64 + e] + before;
      a.slot[((int64_t)t * a.rows + r) * a.k + j] = slot;
      a.perm[t * a.slots + slot] = (int32_t)r;
    }
  }
}

int pt_launch_moe_route(const pt_moe_args& a, hipStream_t s) {
  if (a.rows <= 0 || a.T <= 0) return PT_OK;
  if (a.E < 1 || a.E > 64 || a.k < 1 || a.k > 8 || a.k > a.E || a.slots % 256)
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "expert routing: E = %d, k = %d not covered", a.E, a.k);
  const int64_t n = (int64_t)a.T * a.rows;
  const int nblk = (int)((a.rows + MOE_ROWS - 1) / MOE_ROWS);
  hipLaunchKernelGGL(moe_topk_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a);
  hipLaunchKernelGGL(moe_count_kernel, dim3((unsigned)nblk, (unsigned)a.T), dim3(MOE_ROWS), 0, s, a, nblk);
  hipLaunchKernelGGL(moe_scan_kernel, dim3((unsigned)a.T), dim3(64), 0, s, a, nblk);
  hipLaunchKernelGGL(moe_place_kernel, dim3((unsigned)nblk, (unsigned)a.T), dim3(MOE_ROWS), 0, s, a, nblk);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// ------------------------------------------------------------------------------------------------
// Combine: one workgroup per (row, track).  h = res + sum_j gate_j * y[slot_j], then the RMSNorm that opens the
// next layer.  A thread re-reads only what it wrote itself, so the second pass needs no barrier beyond the one of
// the reduction.
// ------------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) moe_combine_kernel(pt_moe_args a, const float* __restrict__ y, const float* res,
                                                          int64_t res_bstride, float* h, int32_t d,
                                                          const float* __restrict__ gains, int64_t g_bstride, T* out,
                                                          float eps) {
  __shared__ float s_part[4];
  const int64_t r = blockIdx.x;
  const int t = blockIdx.y;
  const int64_t row = (int64_t)t * a.rows + r;
  const int32_t* slot = a.slot + row * a.k;
  const float* gate = a.gate + row * a.k;
  const float4* rsrc = (const float4*)(res + t * res_bstride + r * d);
  float4* hdst = (float4*)(h + row * d);
  const float* yt = y + (int64_t)t * a.slots * d;
  const int n4 = d >> 2;
  float ss = 0.f;
  for (int i = threadIdx.x; i < n4; i += 256) {
    float4 acc = rsrc[i];
    for (int j = 0; j < a.k; ++j) {
      const float g = gate[j];
      const float4 v = ((const float4*)(yt + (int64_t)slot[j] * d))[i];
      acc.x = fmaf(g, v.x, acc.x); acc.y = fmaf(g, v.y, acc.y); acc.z = fmaf(g, v.z, acc.z); acc.w = fmaf(g, v.w, acc.w);
    }
    hdst[i] = acc;
    ss += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
  }
  if (!out) return;
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) s_part[threadIdx.x >> 6] = ss;
  __syncthreads();
  ss = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);
  const float inv = 1.0f / sqrtf(ss / (float)d + eps);
  const float4* g4 = (const float4*)(gains + t * g_bstride);
  T* dst = out + row * d;
  for (int i = threadIdx.x; i < n4; i += 256) {
    const float4 x = hdst[i], w = g4[i];
    elem<T>::st(dst + 4 * i + 0, x.x * inv * w.x);
    elem<T>::st(dst + 4 * i + 1, x.y * inv * w.y);
    elem<T>::st(dst + 4 * i + 2, x.z * inv * w.z);
    elem<T>::st(dst + 4 * i + 3, x.w * inv * w.w);
  }
}

int pt_launch_moe_combine(const pt_moe_args& a, const float* y, const float* res, int64_t res_bstride, float* h,
                          int32_t d, const float* gains, int64_t g_bstride, void* out, int32_t dtype, float eps,
                          hipStream_t s) {
  if (a.rows <= 0 || a.T <= 0) return PT_OK;
  if (d & 3) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "expert combine: d = %d is not a multiple of 4", d);
  dim3 grid((unsigned)a.rows, (unsigned)a.T);
  if (dtype == PT_F32)
    hipLaunchKernelGGL(moe_combine_kernel<float>, grid, dim3(256), 0, s, a, y, res, res_bstride, h, d, gains, g_bstride,
                       (float*)out, eps);
  else
    hipLaunchKernelGGL(moe_combine_kernel<bf16_t>, grid, dim3(256), 0, s, a, y, res, res_bstride, h, d, gains, g_bstride,
                       (bf16_t*)out, eps);
  PT_HIP_CHECK(hipGetLastError());
  return PT_OK;
}

// libpt_ceilings.so: bare loops that measure sustained matrix-core, HBM and LDS rates (include/pt_ceilings.h).
// Benchmark-only translation unit; none of this is on the forward path.
#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma GCC visibility push(default)
#include "pt_ceilings.h"
#pragma GCC visibility pop

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

#define CEIL_CHECK(expr) do { if ((expr) != hipSuccess) return -6; } while (0)

static int device_cus() {
  int dev = 0, v = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 256;
  return v;
}

template <typename F>
static int timed(F&& launch, int reps, hipStream_t st, double* ms_per_launch) {
  hipEvent_t e0, e1;
  CEIL_CHECK(hipEventCreate(&e0));
  CEIL_CHECK(hipEventCreate(&e1));
  launch();   // warm-up
  CEIL_CHECK(hipEventRecord(e0, st));
  for (int i = 0; i < reps; ++i) launch();
  CEIL_CHECK(hipEventRecord(e1, st));
  CEIL_CHECK(hipEventSynchronize(e1));
  CEIL_CHECK(hipGetLastError());
  float ms = 0.f;
  CEIL_CHECK(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  *ms_per_launch = (double)ms / reps;
  return 0;
}

// 16 accumulator tiles (MI = NI = 4) with one wavefront per SIMD, 8 (MI = 2) with two: the register budgets of the
// two GEMM kernel variants.  Two operand sets alternate so that consecutive instructions see different data.
template <int MI, int NI>
__global__ void __launch_bounds__(MI == 4 ? 256 : 512) mfma_loop_kernel(const u32x4_t* __restrict__ src, float* __restrict__ out, int iters) {
  const int tid = threadIdx.x + blockIdx.x * blockDim.x;
  union { u32x4_t u; bf16x8_t v; } a[2][MI], b[2][NI];
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < MI; ++i) a[s][i].u = src[(size_t)(tid * 16 + s * 8 + i) & 0xfffff];
#pragma unroll
    for (int i = 0; i < NI; ++i) b[s][i].u = src[(size_t)(tid * 16 + s * 8 + 4 + i) & 0xfffff];
  }
  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][i].v, b[s][j].v, acc[i][j], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
  out[tid & 0xfffff] = sum;
}

extern "C" int pt_ceiling_mfma_bf16(const void* dev_operands, void* dev_sink, int32_t waves_per_simd, int32_t iters,
                                    int32_t reps, void* hip_stream, double* tflops) {
  if (!dev_operands || !dev_sink || !tflops || iters < 1 || reps < 1 || (waves_per_simd != 1 && waves_per_simd != 2)) return -7;
  hipStream_t st = (hipStream_t)hip_stream;
  const int cus = device_cus();
  double ms = 0;
  int rc;
  if (waves_per_simd == 1)
    rc = timed([&] { hipLaunchKernelGGL((mfma_loop_kernel<4, 4>), dim3(cus), dim3(256), 0, st, (const u32x4_t*)dev_operands, (float*)dev_sink, iters); }, reps, st, &ms);
  else
    rc = timed([&] { hipLaunchKernelGGL((mfma_loop_kernel<2, 4>), dim3(cus), dim3(512), 0, st, (const u32x4_t*)dev_operands, (float*)dev_sink, iters); }, reps, st, &ms);
  if (rc) return rc;
  const double per_wave = waves_per_simd == 1 ? 2.0 * 16 : 2.0 * 8;   // instructions per iteration
  *tflops = (double)cus * 4 * waves_per_simd * iters * per_wave * 32768.0 / (ms * 1e-3) / 1e12;
  return 0;
}

__global__ void __launch_bounds__(256) hbm_read_kernel(const u32x4_t* __restrict__ src, size_t n16, uint32_t* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4_t acc = {0, 0, 0, 0};
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {   // four independent 16-byte loads in flight per lane
    const u32x4_t v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    acc ^= v0 ^ v1 ^ v2 ^ v3;
  }
  for (; i < n16; i += stride) acc ^= src[i];
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[threadIdx.x] = acc.x;   // keeps the loads alive
}

extern "C" int pt_ceiling_hbm_read(const void* dev_src, size_t bytes, void* dev_sink, int32_t reps, void* hip_stream,
                                   double* gbs) {
  if (!dev_src || !dev_sink || !gbs || bytes < (1u << 20) || (bytes & ((1u << 20) - 1)) || reps < 1) return -7;
  hipStream_t st = (hipStream_t)hip_stream;
  *gbs = 0;
  for (int mult : {4, 8, 16, 32, 64}) {   // workgroups per compute unit: the best grid is reported
    const int grid = device_cus() * mult;
    double ms = 0;
    int rc = timed([&] { hipLaunchKernelGGL(hbm_read_kernel, dim3(grid), dim3(256), 0, st, (const u32x4_t*)dev_src, bytes / 16, (uint32_t*)dev_sink); }, reps, st, &ms);
    if (rc) return rc;
    const double r = (double)bytes / (ms * 1e-3) / 1e9;
    if (r > *gbs) *gbs = r;
  }
  return 0;
}

__global__ void __launch_bounds__(256) hbm_copy_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const u32x4_t v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    dst[i] = v0; dst[i + stride] = v1; dst[i + 2 * stride] = v2; dst[i + 3 * stride] = v3;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

extern "C" int pt_ceiling_hbm_copy(const void* dev_src, void* dev_dst, size_t bytes, int32_t reps, void* hip_stream,
                                   double* gbs) {
  if (!dev_src || !dev_dst || !gbs || bytes < (1u << 20) || (bytes & ((1u << 20) - 1)) || reps < 1) return -7;
  hipStream_t st = (hipStream_t)hip_stream;
  *gbs = 0;
  for (int mult : {4, 8, 16, 32, 64}) {
    const int grid = device_cus() * mult;
    double ms = 0;
    int rc = timed([&] { hipLaunchKernelGGL(hbm_copy_kernel, dim3(grid), dim3(256), 0, st, (const u32x4_t*)dev_src, (u32x4_t*)dev_dst, bytes / 16); }, reps, st, &ms);
    if (rc) return rc;
    const double r = 2.0 * (double)bytes / (ms * 1e-3) / 1e9;
    if (r > *gbs) *gbs = r;
  }
  return 0;
}

// 16 reads of 1 KiB per wavefront in flight; 128 KiB of dynamic LDS keep a second workgroup off the compute unit
__global__ void __launch_bounds__(1024) lds_read_kernel(uint32_t* __restrict__ sink, int iters) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 64 * 1024 / 4; i += blockDim.x) ((uint32_t*)smem)[i] = (uint32_t)i;
  __syncthreads();
  u32x4_t acc[16];
#pragma unroll
  for (int u = 0; u < 16; ++u) acc[u] = u32x4_t{0, 0, 0, 0};
  const unsigned char* base = smem + (wave & 3) * 16384 + lane * 16;
  const uint32_t lds_addr = (uint32_t)(uintptr_t)base;
  for (int it = 0; it < iters; ++it) {
    u32x4_t v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v[u]) : "v"(lds_addr), "n"(u * 1024));
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int u = 0; u < 16; ++u) acc[u] ^= v[u];
  }
  u32x4_t s = {0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < 16; ++u) s ^= acc[u];
  sink[(blockIdx.x * blockDim.x + tid) & 0xfffff] = s.x ^ s.y ^ s.z ^ s.w;
}

extern "C" int pt_ceiling_lds_read(void* dev_sink, int32_t waves_per_simd, int32_t iters, int32_t reps, void* hip_stream,
                                   double clock_ghz, double* bytes_per_clk_cu, double* gbs) {
  if (!dev_sink || !bytes_per_clk_cu || !gbs || iters < 1 || reps < 1 || !(clock_ghz > 0) ||
      (waves_per_simd != 1 && waves_per_simd != 2 && waves_per_simd != 4)) return -7;
  hipStream_t st = (hipStream_t)hip_stream;
  static const hipError_t attr = hipFuncSetAttribute((const void*)lds_read_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 128 * 1024);
  if (attr != hipSuccess) return -6;
  const int cus = device_cus(), threads = 256 * waves_per_simd;
  double ms = 0;
  int rc = timed([&] { hipLaunchKernelGGL(lds_read_kernel, dim3(cus), dim3(threads), 128 * 1024, st, (uint32_t*)dev_sink, iters); }, reps, st, &ms);
  if (rc) return rc;
  const double per_cu = (double)threads * 16 * 16 * iters;
  *gbs = per_cu * cus / (ms * 1e-3) / 1e9;
  *bytes_per_clk_cu = per_cu / (ms * 1e-3) / (clock_ghz * 1e9);
  return 0;
}

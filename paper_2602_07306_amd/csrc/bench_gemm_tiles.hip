// libpt_ceilings.so, second part: the prefill GEMM's 256 x 256 tile kernel compiled from the product source with
// phase stamps (PT_GEMM_STAMPS), so that the time of a tile can be split into pipeline fill, K loop, barrier and
// epilogue on the real kernel (include/pt_ceilings.h, bench.py --tile-clocks).  Benchmark-only translation unit.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>
#include <vector>

#define PT_GEMM_STAMPS 1
#include "gemm_mfma_impl.h"

#pragma GCC visibility push(default)
#include "pt_ceilings.h"
#pragma GCC visibility pop

PT_GEMM_INSTANTIATE(EPI_STORE_F32, 0)
PT_GEMM_INSTANTIATE(EPI_RESIDUAL, 0)
PT_GEMM_INSTANTIATE(EPI_SWIGLU, 0)

// the launch helpers report errors through this function of the forward library; here the code is enough
int pt_set_error(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vfprintf(stderr, fmt, ap);
  va_end(ap);
  fputc('\n', stderr);
  return code;
}

#define TILE_CHECK(expr) do { if ((expr) != hipSuccess) return -6; } while (0)

extern "C" int pt_gemm_tile_clocks(int32_t epilogue, const void* dev_a, const void* dev_w, void* dev_out, void* dev_out_bf16,
                                   const float* dev_row_factor, const float* dev_gain, float* dev_row_sums, int32_t M,
                                   int32_t N, int32_t K, int32_t batch, int64_t* dev_stamps, size_t stamp_bytes,
                                   void* hip_stream, double* out10) {
  if (!dev_a || !dev_w || !dev_out || !dev_stamps || !out10) return -2;
  if (M <= 0 || N <= 0 || K < 128 || (K % 128) || batch <= 0 || (M % 256) || (N % 256)) return -2;
  if (epilogue != EPI_STORE_F32 && epilogue != EPI_RESIDUAL && epilogue != EPI_SWIGLU) return -2;
  const int64_t tiles = (int64_t)(M / 256) * (N / 256) * batch;
  const size_t need = (size_t)tiles * 4 * 8 * sizeof(int64_t);
  if (stamp_bytes < need) return -2;
  hipStream_t st = (hipStream_t)hip_stream;
  pt_gemm_args g;
  memset(&g, 0, sizeof(g));
  g.A = (const bf16_t*)dev_a; g.W = (const bf16_t*)dev_w;
  g.a_bstride = (int64_t)M * K; g.w_bstride = (int64_t)N * K; g.lda = K; g.ldb = K;
  g.M = M; g.N = N; g.K = K; g.batch = batch; g.dtype = PT_BF16; g.epi = epilogue;
  g.out = (float*)dev_out; g.out_bstride = (int64_t)M * N; g.ldo = N;
  g.res = (const float*)dev_out; g.res_bstride = (int64_t)M * N;
  g.olp = dev_out; g.olp_bstride = (int64_t)M * (N / 2);
  if (epilogue == EPI_SWIGLU && dev_row_factor) { g.rs_inv = dev_row_factor; g.rs_bstride = M; }
  if (epilogue == EPI_RESIDUAL && dev_out_bf16 && dev_gain && dev_row_sums) {
    g.nf_out = dev_out_bf16; g.nf_out_bstride = (int64_t)M * N;
    g.nf_gain = dev_gain; g.nf_gain_bstride = N;
    g.nf_parts = N / 128;   // one block of sums per wavefront column range of the 256 x 256 tile
    g.nf_ss = dev_row_sums; g.nf_ss_bstride = (int64_t)M * g.nf_parts;
  }
  auto launch = [&]() -> int {
    switch (epilogue) {
      case EPI_STORE_F32: return pt_gemm_mfma_launch_one<EPI_STORE_F32, 0>(g, st);
      case EPI_RESIDUAL: return pt_gemm_mfma_launch_one<EPI_RESIDUAL, 0>(g, st);
      default: return pt_gemm_mfma_launch_one<EPI_SWIGLU, 0>(g, st);
    }
  };
  long long* none = nullptr;
  TILE_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(pt_gemm_stamps), &none, sizeof(none)));
  hipEvent_t e0, e1;
  TILE_CHECK(hipEventCreate(&e0));
  TILE_CHECK(hipEventCreate(&e1));
  if (launch() <= 0) return -6;   // warm-up, no stamps
  TILE_CHECK(hipEventRecord(e0, st));
  for (int i = 0; i < 3; ++i)
    if (launch() <= 0) return -6;
  TILE_CHECK(hipEventRecord(e1, st));
  TILE_CHECK(hipEventSynchronize(e1));
  float ms = 0.f;
  TILE_CHECK(hipEventElapsedTime(&ms, e0, e1));
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  // the stamped launch
  TILE_CHECK(hipMemsetAsync(dev_stamps, 0, need, st));
  long long* stamps = (long long*)dev_stamps;
  TILE_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(pt_gemm_stamps), &stamps, sizeof(stamps)));
  const int rc = launch();
  TILE_CHECK(hipStreamSynchronize(st));
  TILE_CHECK(hipMemcpyToSymbol(HIP_SYMBOL(pt_gemm_stamps), &none, sizeof(none)));
  if (rc <= 0) return -6;
  std::vector<long long> h((size_t)tiles * 32);
  TILE_CHECK(hipMemcpy(h.data(), dev_stamps, need, hipMemcpyDeviceToHost));
  double d[4] = {0, 0, 0, 0}, total = 0, wall = 0;
  long long lo = 0, hi = 0;
  size_t n = 0;
  for (int64_t w = 0; w < tiles * 4; ++w) {
    const long long* t = &h[(size_t)w * 8];
    if (!t[4]) continue;
    for (int i = 0; i < 4; ++i) d[i] += (double)(t[i + 1] - t[i]);
    total += (double)(t[4] - t[0]);
    wall += (double)(t[7] - t[6]);
    if (!n || t[6] < lo) lo = t[6];
    if (!n || t[7] > hi) hi = t[7];
    ++n;
  }
  if (!n) return -6;
  out10[0] = d[0] / n;            // entry to first MFMA, shader clocks
  out10[1] = d[1] / n;            // K loop
  out10[2] = d[2] / n;            // barrier behind the K loop
  out10[3] = d[3] / n;            // epilogue
  out10[4] = total / n;           // whole tile
  out10[5] = wall / n * 10.0;     // whole tile, ns (100 MHz counter)
  out10[6] = (double)(hi - lo) * 10.0;   // first entry to last exit of the launch, ns
  out10[7] = (double)tiles;
  out10[8] = (double)n;           // wavefronts that left stamps
  out10[9] = (double)ms / 3.0;    // ms per launch without stamps (mean of 3)
  return 0;
}

/*
 * pt_ceilings.h - C ABI of libpt_ceilings.so: bare loops that measure what one MI355X sustains, so that a
 * kernel's rate can be read against a measured ceiling next to the published peak (bench.py --ceilings).
 * Not part of the forward library; nothing here computes any step of the model.
 *
 * Every function takes caller-owned device buffers, enqueues `reps` timed launches on the given hipStream_t
 * (NULL = default stream) bracketed by HIP events, synchronises and writes the mean rate of one launch.
 * Returns 0 on success, a negative number on a HIP error or a bad argument.  Nothing is allocated.
 */
#ifndef PT_CEILINGS_H_
#define PT_CEILINGS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Dense bf16 matrix-core loop: every wavefront keeps 16 accumulator tiles of 32x32 and issues
 * v_mfma_f32_32x32x16_bf16 on register operands only (no memory traffic inside the loop), one workgroup of
 * `waves_per_simd` * 4 wavefronts per compute unit (1 or 2).  dev_operands: at least 16 MiB of bf16 values the
 * operands are taken from (all-zero data lets the chip hold its top clock; the model's kind of data does not);
 * dev_sink: at least 4 MiB.  *tflops receives 2*32*32*16 FLOPs per instruction over the launch time. */
int pt_ceiling_mfma_bf16(const void* dev_operands, void* dev_sink, int32_t waves_per_simd, int32_t iters,
                         int32_t reps, void* hip_stream, double* tflops);

/* Streaming read of `bytes` (a multiple of 1 MiB) from dev_src with 16-byte loads, every byte once;
 * dev_sink: at least 4 MiB.  Grids of 4 to 64 workgroups per compute unit are tried; *gbs receives the best
 * bytes / time in GB/s. */
int pt_ceiling_hbm_read(const void* dev_src, size_t bytes, void* dev_sink, int32_t reps, void* hip_stream,
                        double* gbs);

/* Streaming copy of `bytes` (a multiple of 1 MiB) from dev_src to dev_dst; *gbs receives (read + written
 * bytes) / time in GB/s. */
int pt_ceiling_hbm_copy(const void* dev_src, void* dev_dst, size_t bytes, int32_t reps, void* hip_stream,
                        double* gbs);

/* LDS read loop: ds_read_b128 on conflict-free addresses, `waves_per_simd` * 4 wavefronts per compute unit
 * (1, 2 or 4); *bytes_per_clk_cu receives bytes per compute unit per shader clock at clock_ghz (the caller's
 * figure for the clock), *gbs the aggregate rate.  dev_sink: at least 4 MiB. */
int pt_ceiling_lds_read(void* dev_sink, int32_t waves_per_simd, int32_t iters, int32_t reps, void* hip_stream,
                        double clock_ghz, double* bytes_per_clk_cu, double* gbs);

/* Where the time of a 256 x 256 tile of the prefill GEMM goes: one launch of the forward library's tile kernel,
 * compiled from the same source with shader-clock stamps, over batch x ([M, K] x [N, K]^T) in bf16 (M and N
 * multiples of 256, K a multiple of 128).  epilogue: 0 fp32 store, 1 fp32 residual add in place (dev_out), 2 SwiGLU
 * (bf16 [batch][M][N/2] into dev_out).  Optional: dev_row_factor (float [batch][M], SwiGLU: the folded RMSNorm factor),
 * dev_out_bf16 / dev_gain / dev_row_sums (residual: the folded RMSNorm outputs, bf16 [batch][M][N], float
 * [batch][N], float [batch][M][N/128]); all three or none.  dev_stamps: scratch of at least tiles * 4 * 8 * 8 bytes.
 * Three unstamped launches are timed first.  out10: mean shader clocks of entry to first MFMA, K loop, barrier
 * behind it, epilogue, whole tile; then the tile's time in ns, the launch's span in ns, tiles, wavefronts that left
 * stamps, and ms per unstamped launch.  Allocates a host buffer for the stamps only. */
int pt_gemm_tile_clocks(int32_t epilogue, const void* dev_a, const void* dev_w, void* dev_out, void* dev_out_bf16,
                        const float* dev_row_factor, const float* dev_gain, float* dev_row_sums, int32_t M, int32_t N,
                        int32_t K, int32_t batch, int64_t* dev_stamps, size_t stamp_bytes, void* hip_stream,
                        double* out10);

#ifdef __cplusplus
}
#endif
#endif /* PT_CEILINGS_H_ */

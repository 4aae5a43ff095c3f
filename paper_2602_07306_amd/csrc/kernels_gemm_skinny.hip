// Weight-streaming GEMM for decode: C[t] (M x N) = A[t] (M x K) * W[t]^T with M <= 64 rows (one new
// token per sequence).  The work is reading W once from HBM; the matrix cores only keep the arithmetic
// out of the way.
//
// A workgroup owns 32 weight rows (output columns) of one track and all M rows of A; its 4 wavefronts
// split K into four contiguous quarters, so 4 x 32 row streams are in flight per workgroup and even a
// [1024 x 1024] projection spreads over 128 workgroups per track.  The product is formed transposed,
// C^T tile (32 n x 32 m) = W rows (A operand, 16-byte global loads straight into the MFMA layout) times
// A rows (B operand), so a lane owns one row m of C and 4 consecutive columns n per register group.
// The four partial tiles meet in LDS; the fused epilogues (residual add, SwiGLU, RoPE + KV-cache append)
// run on the reduced tile.
//
// The 32 weight rows are two segments of 16: for the paired epilogues the second segment holds the
// partners (up rows of the gate rows; rotary column j + hd/2 of column j), which lands a pair in the
// same lane, registers v and v + 8.
#include "pt_epilogue.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef float f32x4_t __attribute__((ext_vector_type(4)));


struct sk_tile {
  int n_a, n_b;   // first W row of the two 16-row segments
  int j0;         // EPI_QKV / EPI_SWIGLU: first column of the pair inside its head / the FFN
  int qk_head;    // EPI_QKV: head index among the q heads followed by the k heads
  bool rot;       // EPI_QKV: q or k tile (rotary pairs)
};

template <int EPI>
__device__ __forceinline__ sk_tile sk_decode_tile(const pt_gemm_args& g, int tile) {
  sk_tile t;
  t.j0 = 0; t.qk_head = 0; t.rot = false;
  if constexpr (EPI == EPI_SWIGLU) {
    t.j0 = tile * 16;
    t.n_a = swiglu_gate_row(t.j0);
    t.n_b = t.n_a + 32;
  } else if constexpr (EPI == EPI_QKV) {
    const int half_hd = g.hd >> 1, tiles_per_head = half_hd / 16;
    const int rot_tiles = (g.H + g.Hkv) * tiles_per_head;
    t.rot = tile < rot_tiles;
    if (t.rot) {
      t.qk_head = tile / tiles_per_head;
      t.j0 = (tile - t.qk_head * tiles_per_head) * 16;
      t.n_a = t.qk_head * g.hd + t.j0;
      t.n_b = t.n_a + half_hd;
    } else {
      t.n_a = (g.H + g.Hkv) * g.hd + (tile - rot_tiles) * 32;
      t.n_b = t.n_a + 16;
    }
  } else {
    t.n_a = tile * 32;
    t.n_b = t.n_a + 16;
  }
  return t;
}

// MI: 32-row blocks of A (M <= 32*MI); RB: 32-row blocks of W per workgroup (the A fragments of a K batch are
// loaded once and multiplied with RB blocks of weight rows); SK_UNROLL: 16-wide K steps per register batch.
template <int MI, int RB, int EPI, int SK_UNROLL>
__global__ void __launch_bounds__(256) gemm_skinny_kernel(const pt_gemm_args g, int wgs_per_track) {
  __shared__ float red[4][MI][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int b = blockIdx.x / wgs_per_track, wg = blockIdx.x - b * wgs_per_track;

  const int kq = g.K >> 2;   // K quarter of this wavefront
  const bf16_t* wp[RB];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    const sk_tile tl = sk_decode_tile<EPI>(g, wg * RB + rb);
    const int wrow = l32 < 16 ? tl.n_a + l32 : tl.n_b + (l32 - 16);
    wp[rb] = (const bf16_t*)g.W + b * g.w_bstride + (int64_t)wrow * g.ldb + wave * kq + half * 8;
  }
  const bf16_t* ap[MI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
    ap[mi] = (const bf16_t*)g.A + b * g.a_bstride + (int64_t)min(mi * 32 + l32, g.M - 1) * g.lda + wave * kq + half * 8;

  f32x16_t acc[RB][MI];
#pragma unroll
  for (int rb = 0; rb < RB; ++rb)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[rb][mi][v] = 0.f;

  // two register batches of SK_UNROLL K steps: the loads of batch i+1 are in flight while batch i is multiplied
  bf16x8_t wf[2][RB][SK_UNROLL], af[2][SK_UNROLL][MI];
  auto load_batch = [&](int buf, int k) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int u = 0; u < SK_UNROLL; ++u) wf[buf][rb][u] = *(const bf16x8_t*)(wp[rb] + k + 16 * u);
#pragma unroll
    for (int u = 0; u < SK_UNROLL; ++u)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) af[buf][u][mi] = *(const bf16x8_t*)(ap[mi] + k + 16 * u);
  };
  auto mul_batch = [&](int buf) {
#pragma unroll
    for (int u = 0; u < SK_UNROLL; ++u)
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[rb][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[buf][rb][u], af[buf][u][mi], acc[rb][mi], 0, 0, 0);
  };
  constexpr int KB = 16 * SK_UNROLL;
  load_batch(0, 0);
  for (int k = 0; k < kq; k += 2 * KB) {          // kq is a multiple of 2 * KB
    load_batch(1, k + KB);
    mul_batch(0);
    load_batch(0, min(k + 2 * KB, kq - KB));      // past the end: re-read the last batch (unused)
    mul_batch(1);
  }

  // per block of weight rows: reduce the four K quarters through LDS, then the fused epilogue.
  // Register v of a lane is C^T row 8*(v/4) + 4*half + v%4, column l32.  Wavefront w finishes m-block w/2,
  // register groups (w%2) and (w%2)+2: rows 8*(w%2)+4*half+i of each segment.
  const int mi_e = wave >> 1, vg = wave & 1;
  const int m = mi_e * 32 + l32;
  const int off = 8 * vg + 4 * half;   // column offset inside a segment
#pragma unroll
  for (int rb = 0; rb < RB; ++rb) {
    if (rb > 0) __syncthreads();
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) red[wave][mi][v][lane] = acc[rb][mi][v];
    __syncthreads();
    if (mi_e < MI && m < g.M) {
      const sk_tile tl = sk_decode_tile<EPI>(g, wg * RB + rb);
      const int n_a = tl.n_a, n_b = tl.n_b, j0 = tl.j0, qk_head = tl.qk_head;
      float lo[4], hi[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        lo[i] = red[0][mi_e][vg * 4 + i][lane] + red[1][mi_e][vg * 4 + i][lane] + red[2][mi_e][vg * 4 + i][lane] + red[3][mi_e][vg * 4 + i][lane];
        hi[i] = red[0][mi_e][vg * 4 + 8 + i][lane] + red[1][mi_e][vg * 4 + 8 + i][lane] + red[2][mi_e][vg * 4 + 8 + i][lane] + red[3][mi_e][vg * 4 + 8 + i][lane];
      }
      if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_RESIDUAL) {
        float* out = g.out + b * g.out_bstride + (int64_t)m * g.ldo;
        const float* res = EPI == EPI_RESIDUAL ? g.res + b * g.res_bstride + (int64_t)m * g.ldo : nullptr;
#pragma unroll
        for (int sgm = 0; sgm < 2; ++sgm) {
          const int n = (sgm ? n_b : n_a) + off;
          const float* x = sgm ? hi : lo;
          if (n < g.N) {
            f32x4_t v4 = {x[0], x[1], x[2], x[3]};
            if constexpr (EPI == EPI_RESIDUAL) v4 += *(const f32x4_t*)(res + n);
            *(f32x4_t*)(out + n) = v4;
          }
        }
      } else if constexpr (EPI == EPI_SWIGLU) {
        bf16_t* o = (bf16_t*)g.olp + b * g.olp_bstride + (int64_t)m * (g.N >> 1) + j0 + off;
        uint2 pk;
        pk.x = pack_bf16x2(silu_f(lo[0]) * hi[0], silu_f(lo[1]) * hi[1]);
        pk.y = pack_bf16x2(silu_f(lo[2]) * hi[2], silu_f(lo[3]) * hi[3]);
        *(uint2*)o = pk;
      } else {  // EPI_QKV
        const int seq = m / g.S, pos = g.pos0 + (m - seq * g.S);
        const int hd = g.hd, half_hd = hd >> 1, hq = g.H * hd;
        if (tl.rot) {
          const int j = j0 + off;
          const float4* rp = (const float4*)((const float2*)g.rope + (int64_t)pos * half_hd + j);
          const float4 cs01 = rp[0], cs23 = rp[1];
          const float c[4] = {cs01.x, cs01.z, cs23.x, cs23.z}, sn[4] = {cs01.y, cs01.w, cs23.y, cs23.w};
          uint2 plo, phi;
          plo.x = pack_bf16x2(lo[0] * c[0] - hi[0] * sn[0], lo[1] * c[1] - hi[1] * sn[1]);
          plo.y = pack_bf16x2(lo[2] * c[2] - hi[2] * sn[2], lo[3] * c[3] - hi[3] * sn[3]);
          phi.x = pack_bf16x2(hi[0] * c[0] + lo[0] * sn[0], hi[1] * c[1] + lo[1] * sn[1]);
          phi.y = pack_bf16x2(hi[2] * c[2] + lo[2] * sn[2], hi[3] * c[3] + lo[3] * sn[3]);
          bf16_t* dst;
          if (qk_head < g.H) {
            dst = (bf16_t*)g.olp + b * g.olp_bstride + (int64_t)m * hq + qk_head * hd + j;
          } else {
            const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + (qk_head - g.H);
            dst = (bf16_t*)g.kc + hidx * g.kv_head_elems + (int64_t)pos * hd + j;
          }
          *(uint2*)dst = plo;
          *(uint2*)(dst + half_hd) = phi;
        } else {
#pragma unroll
          for (int sgm = 0; sgm < 2; ++sgm) {
            const int cbase = (sgm ? n_b : n_a) - (g.H + g.Hkv) * hd + off;   // column inside the v section
            const float* x = sgm ? hi : lo;
            const int head = cbase / hd, j = cbase - head * hd;
            const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
            bf16_t* vt = (bf16_t*)g.vc + hidx * ((int64_t)hd * g.s_pad) + (int64_t)j * g.s_pad + pos;
#pragma unroll
            for (int i = 0; i < 4; ++i) vt[(int64_t)i * g.s_pad] = f32_to_bf16(x[i]);
          }
        }
      }
    }
  }
}

template <int MI, int RB, int EPI>
static int launch_skinny_rb(const pt_gemm_args& g, int tiles, hipStream_t s) {
  const int wgs = tiles / RB;
  if (g.K % (4 * 16 * 8) == 0)
    hipLaunchKernelGGL((gemm_skinny_kernel<MI, RB, EPI, 4>), dim3((unsigned)(wgs * g.batch)), dim3(256), 0, s, g, wgs);
  else
    hipLaunchKernelGGL((gemm_skinny_kernel<MI, RB, EPI, 2>), dim3((unsigned)(wgs * g.batch)), dim3(256), 0, s, g, wgs);
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

template <int MI, int EPI>
static int launch_skinny(const pt_gemm_args& g, int tiles, hipStream_t s) {
  // more weight-row blocks per workgroup reuse each A fragment more often, as long as enough workgroups remain
  const int64_t wgs1 = (int64_t)tiles * g.batch;
  if (tiles % 4 == 0 && wgs1 / 4 >= 256) return launch_skinny_rb<MI, 4, EPI>(g, tiles, s);
  if (tiles % 2 == 0 && wgs1 / 2 >= 256) return launch_skinny_rb<MI, 2, EPI>(g, tiles, s);
  return launch_skinny_rb<MI, 1, EPI>(g, tiles, s);
}

// Returns 1 if launched, 0 if the shape is not covered.
int pt_launch_gemm_skinny(const pt_gemm_args& g, hipStream_t s) {
  if (g.dtype != PT_BF16 || g.M < 1 || g.M > 64) return 0;
  if (g.K % (4 * 16 * 4) || g.N % 32) return 0;
  if ((g.lda & 7) || (g.ldb & 7) || (g.a_bstride & 7) || (g.w_bstride & 7) || (((uintptr_t)g.A | (uintptr_t)g.W) & 15)) return 0;
  int tiles = g.N / 32;
  if (g.epi == EPI_SWIGLU) {
    if (g.N % 64 || (g.olp_bstride & 3) || ((uintptr_t)g.olp & 7)) return 0;
  } else if (g.epi == EPI_QKV) {
    if (g.hd % 32 || ((g.H + 2 * g.Hkv) * g.hd) != g.N || (g.olp_bstride & 3) || (g.s_pad & 3)) return 0;
  } else {
    if ((g.ldo & 3) || (g.out_bstride & 3) || (g.res_bstride & 3) || (((uintptr_t)g.out | (uintptr_t)g.res) & 15)) return 0;
  }
  if ((int64_t)tiles * g.batch > 0x7fffffff) return 0;
  const bool two = g.M > 32;
  switch (g.epi) {
    case EPI_STORE_F32: return two ? launch_skinny<2, EPI_STORE_F32>(g, tiles, s) : launch_skinny<1, EPI_STORE_F32>(g, tiles, s);
    case EPI_RESIDUAL: return two ? launch_skinny<2, EPI_RESIDUAL>(g, tiles, s) : launch_skinny<1, EPI_RESIDUAL>(g, tiles, s);
    case EPI_SWIGLU: return two ? launch_skinny<2, EPI_SWIGLU>(g, tiles, s) : launch_skinny<1, EPI_SWIGLU>(g, tiles, s);
    case EPI_QKV: return two ? launch_skinny<2, EPI_QKV>(g, tiles, s) : launch_skinny<1, EPI_QKV>(g, tiles, s);
  }
  return 0;
}

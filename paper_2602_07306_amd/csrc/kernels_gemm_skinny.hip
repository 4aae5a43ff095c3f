// Weight-streaming GEMM for decode: C[t] (M x N) = A[t] (M x K) * W[t]^T with M <= 64 rows (one new
// token per sequence).  The work is reading W once from HBM; the matrix cores only keep the arithmetic
// out of the way.
//
// A workgroup owns one to four tiles of 32 weight rows (output columns) of one track and all M rows of A; its
// 4 wavefronts split K (or the workgroup's K slice) into four contiguous ranges.  The product is formed
// transposed, C^T tile (32 n x 32 m) = W rows (MFMA A operand) times A rows (B operand), so a lane owns one
// row m of C and 4 consecutive columns n per register group.  The four partial tiles meet in LDS; the fused
// epilogues (residual add, SwiGLU, RoPE + KV-cache append) run on the reduced tile.  Residual GEMMs with few
// tiles may also split K over workgroups; those leave fp32 slices that the following kernel adds up.
//
// The 32 weight rows are two segments of 16: for the paired epilogues the second segment holds the
// partners (up rows of the gate rows; rotary column j + hd/2 of column j), which lands a pair in the
// same lane, registers v and v + 8.
#include "pt_epilogue.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));


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

// Fused epilogue on the finished (or K-slice) values of row m: lo[i] / hi[i] belong to columns off + i of the
// first / second 16-row segment of `tile` (off a multiple of 4).  ksn > 1 (EPI_RESIDUAL only): slice ks leaves
// its partial product in sk_part[ks][b][m][n]; the kernel that consumes the residual stream adds the slices.
template <int EPI>
__device__ __forceinline__ void sk_finish(const pt_gemm_args& g, int b, int tile, int m, int off, int ks, int ksn,
                                          const float (&lo)[4], const float (&hi)[4]) {
  const sk_tile tl = sk_decode_tile<EPI>(g, tile);
  const int n_a = tl.n_a, n_b = tl.n_b, j0 = tl.j0, qk_head = tl.qk_head;
  (void)n_a; (void)n_b; (void)j0; (void)qk_head;
  if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_RESIDUAL) {
    // K split over workgroups: slice ks leaves its partial product in sk_part[ks][b][m][n]; the kernel that
    // consumes the residual stream adds the slices and the residual
    const bool split = EPI == EPI_RESIDUAL && ksn > 1;
    float* out = split ? g.sk_part + (((int64_t)ks * g.batch + b) * g.M + m) * g.N
                       : g.out + b * g.out_bstride + (int64_t)m * g.ldo;
    const float* res = EPI == EPI_RESIDUAL ? g.res + b * g.res_bstride + (int64_t)m * g.ldo : nullptr;
#pragma unroll
    for (int sgm = 0; sgm < 2; ++sgm) {
      const int n = (sgm ? n_b : n_a) + off;
      const float* x = sgm ? hi : lo;
      if (n < g.N) {
        f32x4_t v4 = {x[0], x[1], x[2], x[3]};
        if constexpr (EPI == EPI_RESIDUAL) if (!split) v4 += *(const f32x4_t*)(res + n);
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
    const pt_rowpos rp = gemm_row_pos(g, m);
    const int seq = rp.seq, pos = rp.pos;
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

// MI: 32-row blocks of A (M <= 32*MI); RB: 32-row blocks of W per workgroup (each A fragment is multiplied
// with RB blocks of weight rows).
//
// K advances in steps of 64 per wavefront.  Both operands are read from global memory as whole 128-byte row
// pieces (8 lanes per row, 8 rows per load instruction): lane-per-row loads in the MFMA operand layout touch
// 32 cache lines per instruction and hold the vector-memory path below what HBM delivers.  The pieces are
// parked in LDS private to the wavefront and picked up from there as MFMA fragments.  Row r of a parked
// block holds its 16-byte chunk c at position c ^ swizzle(r): writes and fragment reads are conflict-free.
// Weight rows use two rotating register sets, refilled with step s+2 as soon as step s is parked, so two
// steps of weights are in flight per wavefront; A uses one register set and one LDS slot.
// `items` > 1: the workgroup works through that many consecutive groups of RB tiles of its track, and the first
// loads of the next group are in flight while the partial tiles of the current one are reduced and stored.  All
// workgroups of a launch start together; with one group each they would all wait for their first loads, stream,
// and reduce at the same moments, and HBM would idle in between.
template <int MI, int RB, int EPI>
__device__ __forceinline__ void skinny_body(const pt_gemm_args& g, int b, int first_tile, int ks, int ksn, int items = 1) {
  constexpr int A_STEP = MI * 32 * 128;                 // bytes of A per K step
  constexpr int W_STEP = RB * 32 * 128;                 // bytes of W per K step
  constexpr int RING = A_STEP + W_STEP;                 // per wavefront
  extern __shared__ __attribute__((aligned(1024))) char smem[];   // max(4 * RING, reduction buffer) bytes
  float (*red)[MI][16][64] = (float (*)[MI][16][64])smem;         // reuses the rings after the K loop
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int kq = g.K / (4 * ksn);   // K range of this wavefront, a multiple of 128
  const int k_first = (ks * 4 + wave) * kq;
  const int nsteps = kq >> 6;

  // staging: load i of a 32-row block brings rows 8i .. 8i+7, lane L the chunk L%8 of row 8i + L/8
  auto swz = [](int row) { return (row >> 1) & 7; };
  char* a_ring = smem + wave * RING;
  char* w_slot = a_ring + A_STEP;
  int dst[4];   // position inside a parked 32-row block
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = i * 8 + (lane >> 3);
    dst[i] = row * 128 + (((lane & 7) ^ swz(row)) * 16);
  }
  const bf16_t* w_src[RB][4];
  auto set_w_src = [&](int tile0) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      const sk_tile tl = sk_decode_tile<EPI>(g, tile0 + rb);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int r = i * 8 + (lane >> 3);
        const int wrow = r < 16 ? tl.n_a + r : tl.n_b + (r - 16);
        w_src[rb][i] = (const bf16_t*)g.W + b * g.w_bstride + (int64_t)wrow * g.ldb + k_first + (lane & 7) * 8;
      }
    }
  };
  set_w_src(first_tile);
  const bf16_t* a_src[4 * MI];
#pragma unroll
  for (int j = 0; j < 4 * MI; ++j) {
    const int row = j * 8 + (lane >> 3);
    const int mrow = min(row, g.M - 1);
    const int64_t arow = g.a_rows ? g.a_rows[b * g.a_rows_bstride + mrow] : mrow;   // grouped GEMM: gathered rows
    a_src[j] = (const bf16_t*)g.A + b * g.a_bstride + arow * g.lda + k_first + (lane & 7) * 8;
  }
  u32x4_t areg[4 * MI], wreg[2][RB][4];
  auto load_a = [&](int step) {
#pragma unroll
    for (int j = 0; j < 4 * MI; ++j) areg[j] = *(const u32x4_t*)(a_src[j] + step * 64);
  };
  auto park_a = [&](int step) {
    char* slot = a_ring;
    (void)step;
#pragma unroll
    for (int j = 0; j < 4 * MI; ++j) *(u32x4_t*)(slot + (j >> 2) * 4096 + dst[j & 3]) = areg[j];
  };
  auto load_w = [&](int buf, int step) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 4; ++i) wreg[buf][rb][i] = *(const u32x4_t*)(w_src[rb][i] + step * 64);
  };
  auto park_w = [&](int buf) {
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int i = 0; i < 4; ++i) *(u32x4_t*)(w_slot + rb * 4096 + dst[i]) = wreg[buf][rb][i];
  };
  // fragment of a 32-row block for K sub-step u (16 wide): row l32, chunk 2u + half
  const int fr_row = l32 * 128, fr_sw = swz(l32);

  f32x16_t acc[RB][MI];

  auto mul_step = [&](int step) {
    const char* a_slot = a_ring;
    (void)step;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int fo = fr_row + (((2 * u + half) ^ fr_sw) * 16);
      bf16x8_t af[MI], wfr[RB];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) af[mi] = *(const bf16x8_t*)(a_slot + mi * 4096 + fo);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb) wfr[rb] = *(const bf16x8_t*)(w_slot + rb * 4096 + fo);
#pragma unroll
      for (int rb = 0; rb < RB; ++rb)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[rb][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[rb], af[mi], acc[rb][mi], 0, 0, 0);
    }
  };

  // Loads past the last step re-read it (never used).  The prologue issues its loads in the order of the
  // loop body, so that the waits the compiler derives for the loop need not cover a different order on entry.
  // Register v of a lane is C^T row 8*(v/4) + 4*half + v%4, column l32.  Wavefront w finishes m-block w/2,
  // register groups (w%2) and (w%2)+2: rows 8*(w%2)+4*half+i of each segment.
  const int mi_e = wave >> 1, vg = wave & 1;
  const int m = mi_e * 32 + l32;
  const int off = 8 * vg + 4 * half;   // column offset inside a segment
  const bool owner = mi_e < MI && m < g.M;

  load_w(0, 0);
  __builtin_amdgcn_sched_barrier(0);
  load_a(0);
  for (int item = 0; item < items; ++item) {
    const int tile0 = first_tile + item * RB;
#pragma unroll
    for (int rb = 0; rb < RB; ++rb)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[rb][mi][v] = 0.f;
    __builtin_amdgcn_sched_barrier(0);
    park_a(0);
    __builtin_amdgcn_sched_barrier(0);
    load_w(1, min(1, nsteps - 1));
    __builtin_amdgcn_sched_barrier(0);
    load_a(min(1, nsteps - 1));
    for (int s0 = 0; s0 < nsteps; s0 += 2) {   // nsteps is even
#pragma unroll
      for (int par = 0; par < 2; ++par) {
        const int st = s0 + par;
        __builtin_amdgcn_sched_barrier(0);
        park_w(par);                                // step st; the fragments of step st-1 have been read
        __builtin_amdgcn_sched_barrier(0);
        load_w(par, min(st + 2, nsteps - 1));
        __builtin_amdgcn_sched_barrier(0);
        mul_step(st);
        __builtin_amdgcn_sched_barrier(0);
        park_a(st + 1);                             // the fragments of step st have been read
        __builtin_amdgcn_sched_barrier(0);
        load_a(min(st + 2, nsteps - 1));
      }
    }
    __syncthreads();   // the rings become the reduction buffer
    if (item + 1 < items) {
      // the next group's first loads travel while this one is reduced and stored
      __builtin_amdgcn_sched_barrier(0);
      set_w_src(tile0 + RB);
      load_w(0, 0);
      __builtin_amdgcn_sched_barrier(0);
      load_a(0);
      __builtin_amdgcn_sched_barrier(0);
    }

    // per block of weight rows: the four wavefronts' partial tiles meet in LDS
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
      if (rb > 0) __syncthreads();
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) red[wave][mi][v][lane] = acc[rb][mi][v];
      __syncthreads();
      if (owner) {
        float lo[4], hi[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          lo[i] = red[0][mi_e][vg * 4 + i][lane] + red[1][mi_e][vg * 4 + i][lane] + red[2][mi_e][vg * 4 + i][lane] + red[3][mi_e][vg * 4 + i][lane];
          hi[i] = red[0][mi_e][vg * 4 + 8 + i][lane] + red[1][mi_e][vg * 4 + 8 + i][lane] + red[2][mi_e][vg * 4 + 8 + i][lane] + red[3][mi_e][vg * 4 + 8 + i][lane];
        }
        sk_finish<EPI>(g, b, tile0 + rb, m, off, ks, ksn, lo, hi);
      }
    }
    if (item + 1 < items) __syncthreads();   // the reduction buffer becomes the rings again
  }
}

// ------------------------------------------------------------------------------------------------
// M <= 4 rows (latency-mode decode, one to four sequences): matrix-vector form on the vector ALUs.
// Nothing is staged: a wavefront reads 8 weight rows (4 epilogue pairs of a 32-row tile) as 1 KB
// contiguous pieces, 16 bytes per lane, multiplies them with the A values of the lane's K positions
// (A sits in LDS, bf16) and folds the 64 lanes with cross-lane adds at the end.  Two register sets keep
// 16 KB of weights in flight per wavefront.  A workgroup (4 wavefronts) owns one 32-row tile.
// ------------------------------------------------------------------------------------------------
template <int MR, int EPI>
__global__ void __launch_bounds__(256) gemm_gemv_kernel(const pt_gemm_args g, int tiles, int wgs_per_track) {
  extern __shared__ __attribute__((aligned(16))) char smem[];   // A: [MR][K] bf16
  bf16_t* As = (bf16_t*)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b = blockIdx.x / wgs_per_track, wg = blockIdx.x - b * wgs_per_track;
  const int K = g.K;
  // A rows into LDS (rows past M repeat the last one; their results are not stored)
  if (g.norm_src) {
    // A = RMSNorm of the fp32 residual stream, formed here (every workgroup repeats these few thousand
    // operations; the launch of a separate kernel would cost more)
    __shared__ float s_ss[4];
    const float* gain = g.norm_gain + b * g.norm_gbstride;
    for (int m = 0; m < MR; ++m) {
      const float* x = g.norm_src + b * g.norm_bstride + (int64_t)min(m, g.M - 1) * K;
      float ss = 0.f;
      for (int k4 = tid; k4 < (K >> 2); k4 += 256) {
        const f32x4_t v = *(const f32x4_t*)(x + 4 * k4);
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
      }
      ss = wave_sum(ss);
      if (m > 0) __syncthreads();
      if (lane == 0) s_ss[wave] = ss;
      __syncthreads();
      ss = (s_ss[0] + s_ss[1]) + (s_ss[2] + s_ss[3]);
      const float inv = 1.0f / sqrtf(ss / (float)K + g.norm_eps);
      for (int k4 = tid; k4 < (K >> 2); k4 += 256) {
        const f32x4_t v = *(const f32x4_t*)(x + 4 * k4);
        const f32x4_t w = *(const f32x4_t*)(gain + 4 * k4);
        uint2 pk;
        pk.x = pack_bf16x2(v.x * inv * w.x, v.y * inv * w.y);
        pk.y = pack_bf16x2(v.z * inv * w.z, v.w * inv * w.w);
        *(uint2*)(As + m * K + 4 * k4) = pk;
      }
    }
  } else {
    for (int c = tid; c < MR * (K >> 3); c += 256) {
      const int m = c / (K >> 3), kc = c - m * (K >> 3);
      *(u32x4_t*)(As + m * K + kc * 8) =
          *(const u32x4_t*)((const bf16_t*)g.A + b * g.a_bstride + (int64_t)min(m, g.M - 1) * g.lda + kc * 8);
    }
  }
  // This workgroup's tiles: wg, wg + wgs_per_track, ...  The wavefront walks (tile, 512-wide K chunk) items
  // in one stream, so the loads of a tile's first chunks are in flight while the previous tile is finished.
  const int my_tiles = (tiles - wg + wgs_per_track - 1) / wgs_per_track;
  const int nchunks = K >> 9;   // K is a multiple of 512
  const int nitems = my_tiles * nchunks;
  const bf16_t* wrow[8];   // rows 2i: first segment, 2i + 1: partner in the second segment
  auto set_rows = [&](int tile) {
    const sk_tile tl = sk_decode_tile<EPI>(g, tile);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int p = wave * 4 + i;
      wrow[2 * i] = (const bf16_t*)g.W + b * g.w_bstride + (int64_t)(tl.n_a + p) * g.ldb + lane * 8;
      wrow[2 * i + 1] = (const bf16_t*)g.W + b * g.w_bstride + (int64_t)(tl.n_b + p) * g.ldb + lane * 8;
    }
  };
  float acc[8][MR];
#pragma unroll
  for (int r = 0; r < 8; ++r)
#pragma unroll
    for (int m = 0; m < MR; ++m) acc[r][m] = 0.f;
  u32x4_t wreg[2][8];
  int ld_tile = wg, ld_chunk = 0;    // the load stream's position
  set_rows(ld_tile);
  auto load_next = [&](int buf) {     // past the last item: re-reads the last chunk (unused)
#pragma unroll
    for (int r = 0; r < 8; ++r) wreg[buf][r] = *(const u32x4_t*)(wrow[r] + ld_chunk * 512);
    if (ld_chunk + 1 < nchunks) {
      ++ld_chunk;
    } else if (ld_tile + wgs_per_track < tiles) {
      ld_tile += wgs_per_track;
      ld_chunk = 0;
      set_rows(ld_tile);
    }
  };
  int cur_tile = wg, cur_chunk = 0;  // the multiply stream's position
  auto mul = [&](int buf) {
    float av[MR][8];
#pragma unroll
    for (int m = 0; m < MR; ++m) {
      const u32x4_t a4 = *(const u32x4_t*)(As + m * K + cur_chunk * 512 + lane * 8);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        av[m][2 * i] = __uint_as_float(a4[i] << 16);
        av[m][2 * i + 1] = __uint_as_float(a4[i] & 0xffff0000u);
      }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w0 = __uint_as_float(wreg[buf][r][i] << 16), w1 = __uint_as_float(wreg[buf][r][i] & 0xffff0000u);
#pragma unroll
        for (int m = 0; m < MR; ++m) acc[r][m] = fmaf(w1, av[m][2 * i + 1], fmaf(w0, av[m][2 * i], acc[r][m]));
      }
    if (++cur_chunk == nchunks) {     // the tile is complete: fold the lanes, lane m finishes A row m
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int m = 0; m < MR; ++m) acc[r][m] = wave_sum(acc[r][m]);
#pragma unroll
      for (int m = 0; m < MR; ++m) {
        if (lane == m && m < g.M) {
          const float lo[4] = {acc[0][m], acc[2][m], acc[4][m], acc[6][m]};
          const float hi[4] = {acc[1][m], acc[3][m], acc[5][m], acc[7][m]};
          sk_finish<EPI>(g, b, cur_tile, m, wave * 4, 0, 1, lo, hi);
        }
      }
#pragma unroll
      for (int r = 0; r < 8; ++r)
#pragma unroll
        for (int m = 0; m < MR; ++m) acc[r][m] = 0.f;
      cur_tile += wgs_per_track;
      cur_chunk = 0;
    }
  };
  load_next(0);
  __syncthreads();              // A is in LDS
  for (int i = 0; i < nitems; i += 2) {
    __builtin_amdgcn_sched_barrier(0);
    load_next(1);
    __builtin_amdgcn_sched_barrier(0);
    mul(0);
    __builtin_amdgcn_sched_barrier(0);
    load_next(0);
    __builtin_amdgcn_sched_barrier(0);
    if (i + 1 < nitems) mul(1);
  }
}

template <int MR, int EPI>
static int launch_gemv(const pt_gemm_args& g, int tiles, hipStream_t s) {
  const int lds = MR * g.K * 2;
  auto kern = gemm_gemv_kernel<MR, EPI>;
  PT_SET_MAX_LDS_ONCE(kern, 48 * 1024);
  // about a thousand workgroups (three to four resident per compute unit), every one with the same number of tiles
  const int tpw = (int)(((int64_t)tiles * g.batch + 1023) / 1024);
  const int wpt = (tiles + tpw - 1) / tpw;
  hipLaunchKernelGGL(kern, dim3((unsigned)((int64_t)wpt * g.batch)), dim3(256), lds, s, g, tiles, wpt);
  PT_HIP_CHECK(hipGetLastError());
  return 3;
}

template <int EPI>
static int launch_gemv_m(const pt_gemm_args& g, int tiles, hipStream_t s) {
  if (g.M == 1) return launch_gemv<1, EPI>(g, tiles, s);
  if (g.M == 2) return launch_gemv<2, EPI>(g, tiles, s);
  return launch_gemv<4, EPI>(g, tiles, s);
}

// Grouped GEMM (rows grouped by weight matrix, e.g. the experts of a PT-MoE layer): the batch index of the grid runs
// over (track, group); a workgroup works on the rows of its group only, through a view of the arguments whose
// pointers start at the group's first row.  Groups without rows are skipped, their weights never read.
template <int MI, int RB, int EPI>
__device__ __forceinline__ void skinny_group(const pt_gemm_args& g, int bg, int first_tile, int ks, int ksn) {
  const int t = bg / g.n_groups, e = bg - t * g.n_groups;
  const int count = g.grp_count[t * g.grp_info_bstride + e];
  if (count <= 0) return;
  const int base = g.grp_base[t * g.grp_info_bstride + e];
  pt_gemm_args v = g;
  v.M = min(count, 32 * MI);
  v.W = (const bf16_t*)g.W + t * g.w_bstride + e * g.w_gstride;
  v.A = (const bf16_t*)g.A + t * g.a_bstride + (g.a_rows ? 0 : (int64_t)base * g.lda);
  v.a_rows = g.a_rows ? g.a_rows + t * g.a_rows_bstride + base : nullptr;
  if constexpr (EPI == EPI_SWIGLU) v.olp = (bf16_t*)g.olp + t * g.olp_bstride + (int64_t)base * (g.N >> 1);
  else v.out = g.out + t * g.out_bstride + (int64_t)base * g.ldo;
  skinny_body<MI, RB, EPI>(v, 0, first_tile, ks, ksn);
}

template <int MI, int RB, int EPI>
__device__ __forceinline__ void skinny_dispatch(const pt_gemm_args& g, int b, int first_tile, int ks, int ksn, int items = 1) {
  if constexpr (EPI == EPI_SWIGLU || EPI == EPI_STORE_F32) {
    if (g.n_groups > 0) { skinny_group<MI, RB, EPI>(g, b, first_tile, ks, ksn); return; }   // one group of tiles each
  }
  skinny_body<MI, RB, EPI>(g, b, first_tile, ks, ksn, items);
}

// The tiles (blocks of 32 weight rows) of a track are dealt out to wgs_per_track workgroups as evenly as
// possible: `rem` workgroups take RBHI tiles, the others RBHI - 1 (all take RBHI when rem == 0).  The grid
// lists the larger workgroups of all tracks first, so that a second round of workgroups fills up evenly.
// Workgroups that share output tiles (one per K slice, EPI_RESIDUAL only) are neighbours in the grid.
// items > 1 (only with rem == 0): wgs_per_track counts workgroups that take `items` consecutive groups of RBHI tiles.
template <int MI, int RBHI, int EPI>
__global__ void __launch_bounds__(256) gemm_skinny_kernel(const pt_gemm_args g, int wgs_per_track, int rem, int ksn, int items) {
  const int unit = blockIdx.x / ksn, ks = blockIdx.x - unit * ksn;
  if (rem == 0) {
    const int b = unit / wgs_per_track, wg = unit - b * wgs_per_track;
    skinny_dispatch<MI, RBHI, EPI>(g, b, wg * items * RBHI, ks, ksn, items);
    return;
  }
  const int n_big = rem * g.batch;
  if (unit < n_big) {
    const int b = unit / rem, wg = unit - b * rem;
    skinny_dispatch<MI, RBHI, EPI>(g, b, wg * RBHI, ks, ksn);
  } else {
    if constexpr (RBHI > 1) {
      const int small = wgs_per_track - rem, u2 = unit - n_big;
      const int b = u2 / small, wg = u2 - b * small;
      skinny_dispatch<MI, RBHI - 1, EPI>(g, b, rem * RBHI + wg * (RBHI - 1), ks, ksn);
    }
  }
}

// Tuning knob for benchmarks (pt_set_tuning): 0 = automatic, else 256 * workgroups per track + K slices
// (where the shape allows).
int pt_tune_skinny_plan = 0;
static int pt_tune_skinny_items = 0;   // 0: automatic; 1: one group of tiles per workgroup; n: n groups where the plan allows

struct sk_plan { int wpt, ks; };

static int device_cus();

template <int MI, int RBHI, int EPI>
static int launch_skinny_rb(const pt_gemm_args& g, int tiles, sk_plan p, hipStream_t s) {
  constexpr int RING = 4 * (MI + RBHI) * 32 * 128, RED = 4 * MI * 16 * 64 * 4;
  constexpr int LDS = RING > RED ? RING : RED;
  // Groups of tiles per workgroup: when every workgroup takes the same number of tiles, as many consecutive groups
  // as still leave every compute unit its resident workgroups (LDS: 160 KB per compute unit).
  int items = 1;
  if (tiles % p.wpt == 0 && g.n_groups == 0 && pt_tune_skinny_items != 1) {
    const int64_t total = (int64_t)p.wpt * g.batch * p.ks;
    const int64_t resident = (int64_t)device_cus() * ((160 * 1024) / LDS >= 3 ? 3 : (160 * 1024) / LDS >= 2 ? 2 : 1);
    for (int d = 2; d <= 16; ++d)
      if (p.wpt % d == 0 && total / d >= resident) items = d;
    if (pt_tune_skinny_items > 1 && p.wpt % pt_tune_skinny_items == 0) items = pt_tune_skinny_items;
  }
  const int wpt = p.wpt / items;
  const unsigned grid = (unsigned)((int64_t)wpt * g.batch * p.ks);
  auto kern = gemm_skinny_kernel<MI, RBHI, EPI>;
  PT_SET_MAX_LDS_ONCE(kern, LDS);
  hipLaunchKernelGGL(kern, dim3(grid), dim3(256), LDS, s, g, wpt, tiles % p.wpt, p.ks, items);
  PT_HIP_CHECK(hipGetLastError());
  return 2;
}

static int device_cus() {
  static int n = 0;
  if (!n) {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
      n = v;
    else
      n = 256;
  }
  return n;
}

// Workgroups per track and K slices.  One workgroup is resident per compute unit (LDS), so the grid runs in
// rounds of n_cu workgroups; a workgroup's time grows with its K steps (plus a fixed start-up and reduction
// cost of about six steps) and with the rows it loads per step (its tiles of W plus the shared A rows).
// K slices (ks_max > 1: residual GEMMs whose caller adds the slices) shorten the rounds of shapes with few tiles.
static sk_plan plan_skinny(const pt_gemm_args& g, int tiles, int ks_max) {
  const int n_cu = device_cus();
  const double a_rows = g.M > 32 ? 0.6 : 0.3;
  sk_plan best = {(tiles + 3) / 4, 1};
  double best_cost = 1e30;
  for (int ks = 1; ks <= ks_max; ++ks) {
    if (g.K % (ks * 4 * 128)) continue;                          // an even number of K steps per wavefront
    if (ks > 1 && (int64_t)ks * g.batch * g.M * g.N > g.sk_part_floats) break;
    const double steps = g.K / (ks * 256) + 6.0;
    const int wpt_min = (tiles + 3) / 4;
    // candidates: the fewest workgroups, and the grids that fill whole rounds
    int cand[6], nc = 0;
    cand[nc++] = wpt_min;
    cand[nc++] = (tiles + 1) / 2;
    cand[nc++] = tiles;
    const int64_t per_round = n_cu;   // workgroups of all tracks and slices in a round
    for (int rounds = 1; rounds <= 3; ++rounds) {
      const int64_t w = per_round * rounds / ((int64_t)g.batch * ks);
      if (w >= wpt_min && w <= tiles && w * g.batch * ks == per_round * rounds) cand[nc++] = (int)w;
    }
    for (int i = 0; i < nc; ++i) {
      const int wpt = cand[i];
      const int rb_hi = (tiles + wpt - 1) / wpt;
      const int64_t wgs = (int64_t)wpt * g.batch * ks;
      const int64_t rounds = (wgs + n_cu - 1) / n_cu;
      const double cost = rounds * steps * (rb_hi + a_rows);
      if (cost < best_cost * 0.999) { best_cost = cost; best.wpt = wpt; best.ks = ks; }
    }
  }
  if (pt_tune_skinny_plan > 0) {
    const int fw = pt_tune_skinny_plan >> 8, fks = pt_tune_skinny_plan & 255;
    if (fw >= (tiles + 3) / 4 && fw <= tiles) best.wpt = fw;
    best.ks = 1;
    if (fks > 1 && fks <= ks_max && g.K % (fks * 4 * 128) == 0 && (int64_t)fks * g.batch * g.M * g.N <= g.sk_part_floats)
      best.ks = fks;
  }
  return best;
}

template <int MI, int EPI>
static int launch_skinny(const pt_gemm_args& g, int tiles, int ks_max, hipStream_t s) {
  const sk_plan p = plan_skinny(g, tiles, ks_max);
  switch ((tiles + p.wpt - 1) / p.wpt) {
    case 4: return launch_skinny_rb<MI, 4, EPI>(g, tiles, p, s);
    case 3: return launch_skinny_rb<MI, 3, EPI>(g, tiles, p, s);
    case 2: return launch_skinny_rb<MI, 2, EPI>(g, tiles, p, s);
    default: return launch_skinny_rb<MI, 1, EPI>(g, tiles, p, s);
  }
}

static bool skinny_covers(const pt_gemm_args& g) {
  if (g.dtype != PT_BF16 || g.M < 1 || g.M > 64) return false;
  if (g.K % (4 * 128) || g.N % 32) return false;
  if ((g.lda & 7) || (g.ldb & 7) || (g.a_bstride & 7) || (g.w_bstride & 7) || (((uintptr_t)g.A | (uintptr_t)g.W) & 15)) return false;
  const int tiles = g.N / 32;
  if (g.epi == EPI_SWIGLU) {
    if (g.N % 64 || (g.olp_bstride & 3) || ((uintptr_t)g.olp & 7)) return false;
  } else if (g.epi == EPI_QKV) {
    if (g.hd % 32 || ((g.H + 2 * g.Hkv) * g.hd) != g.N || (g.olp_bstride & 3) || (g.s_pad & 3)) return false;
  } else {
    if ((g.ldo & 3) || (g.out_bstride & 3) || (g.res_bstride & 3) || (((uintptr_t)g.out | (uintptr_t)g.res) & 15)) return false;
  }
  return (int64_t)tiles * g.batch * 16 <= 0x7fffffff;
}

// Number of K slices the decode kernel would use for this residual GEMM when the caller is ready to add the
// slices itself (0: the kernel does not cover the shape; 1: no split).
// one to four rows: matrix-vector kernel, if A fits its LDS budget and the grid is at least half a round
static bool use_gemv(const pt_gemm_args& g) {
  return g.M <= 4 && g.n_groups == 0 && pt_tune_skinny_plan == 0 && g.K % 512 == 0 &&
         (int64_t)(g.M == 3 ? 4 : g.M) * g.K * 2 <= 48 * 1024 && (int64_t)(g.N / 32) * g.batch >= 128;
}

bool pt_gemm_fuses_norm(const pt_gemm_args& g) {
  return skinny_covers(g) && use_gemv(g) && (g.epi == EPI_QKV || g.epi == EPI_SWIGLU) && g.lda == g.K;
}

int pt_gemm_skinny_ksplit(const pt_gemm_args& g) {
  if (!skinny_covers(g)) return 0;
  if (g.epi != EPI_RESIDUAL || !g.sk_part || (g.N & 3) || use_gemv(g)) return 1;
  return plan_skinny(g, g.N / 32, 16).ks;
}

// Returns the kernel family launched (2, or 3 for the matrix-vector form), 0 if the shape is not covered.  With allow_split the K slices chosen by
// pt_gemm_skinny_ksplit are left in g.sk_part instead of the finished residual stream.
int pt_launch_gemm_skinny(const pt_gemm_args& g_in, bool allow_split, hipStream_t s) {
  pt_gemm_args g = g_in;
  if (g.n_groups > 0) {
    // grouped: one batch entry per (track, group), each with at most grp_max_rows rows
    if (g.grp_max_rows > 64 || !g.grp_count || !g.grp_base || (g.w_gstride & 7)) return 0;
    if (g.epi != EPI_SWIGLU && g.epi != EPI_STORE_F32) return 0;
    g.M = g.grp_max_rows;
    g.batch = g_in.batch * g.n_groups;
    allow_split = false;
  }
  if (!skinny_covers(g)) return 0;
  const int tiles = g.N / 32;
  const int ks_max = allow_split && g.epi == EPI_RESIDUAL && g.sk_part && !(g.N & 3) ? 16 : 1;
  if (g.norm_src && !pt_gemm_fuses_norm(g)) return 0;
  if (use_gemv(g)) {
    switch (g.epi) {
      case EPI_STORE_F32: return launch_gemv_m<EPI_STORE_F32>(g, tiles, s);
      case EPI_RESIDUAL: return launch_gemv_m<EPI_RESIDUAL>(g, tiles, s);
      case EPI_SWIGLU: return launch_gemv_m<EPI_SWIGLU>(g, tiles, s);
      case EPI_QKV: return launch_gemv_m<EPI_QKV>(g, tiles, s);
    }
  }
  const bool two = g.M > 32;
  switch (g.epi) {
    case EPI_STORE_F32: return two ? launch_skinny<2, EPI_STORE_F32>(g, tiles, ks_max, s) : launch_skinny<1, EPI_STORE_F32>(g, tiles, ks_max, s);
    case EPI_RESIDUAL: return two ? launch_skinny<2, EPI_RESIDUAL>(g, tiles, ks_max, s) : launch_skinny<1, EPI_RESIDUAL>(g, tiles, ks_max, s);
    case EPI_SWIGLU: return two ? launch_skinny<2, EPI_SWIGLU>(g, tiles, ks_max, s) : launch_skinny<1, EPI_SWIGLU>(g, tiles, ks_max, s);
    case EPI_QKV: return two ? launch_skinny<2, EPI_QKV>(g, tiles, ks_max, s) : launch_skinny<1, EPI_QKV>(g, tiles, ks_max, s);
  }
  return 0;
}

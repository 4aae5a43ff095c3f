// Track-batched bf16 GEMM on the gfx950 matrix cores with fused epilogues.
//
//   C[t] (M x N) = A[t] (M x K) * W[t]^T,   W[t] stored [N, K], for every track t (grid z-like dim)
//
// Both operands are contiguous along K, so a lane's 8-element MFMA operand is one 16-byte LDS read.
// Tiling: a workgroup owns a BM x BN tile; WM x WN wavefronts each own a (BM/WM) x (BN/WN) sub-tile
// made of 32x32x16 MFMAs.  K advances in steps of 64 through a double-buffered LDS tile whose
// 16-byte chunks are XOR-swizzled by the row number, so that neither the 16-byte stores (8 lanes per
// row) nor the operand reads (32 consecutive rows per half-wave) pile onto the same banks.  Global
// loads for step k+1 are issued before the MFMAs of step k and parked in registers.
//
// Accumulator layout of a 32x32 MFMA tile: lane l holds column l%32 and, in register v, row
// 8*(v/4) + 4*(l/32) + v%4.  The epilogues work directly on that layout:
//   - fp32 stores / residual adds are 128-byte row segments per register;
//   - the SwiGLU pair (gate_j, up_j) is (tile ni, tile ni+1) in the same lane and register, because
//     the weight rows are interleaved in blocks of 32;
//   - the rotary pair (j, j + hd/2) is (tile ni, tile ni + hd/64) in the same lane and register;
//   - V is written transposed: 4 consecutive rows of a register group are 4 consecutive positions.
#include "pt_epilogue.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // 16-byte staging register

#define GM_BK 64
#ifndef GM_SWZ
#define GM_SWZ(row) (((row) >> 1) & 7)
#endif

struct tile_coord {
  int b, tm, tn;
};

// Workgroup id -> (track, m-tile, n-tile).  Consecutive ids are dealt round-robin to the 8 XCDs, so
// ids are first regrouped so that each XCD (own L2) walks a contiguous range; inside a range, tiles
// are visited in groups of 4 m-tiles x all n-tiles, column-major inside the group, which keeps the
// A and W slabs of concurrently resident workgroups few.
__device__ __forceinline__ tile_coord map_tile(int id, int total, int tiles_m, int tiles_n) {
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int per_b = tiles_m * tiles_n;
  tile_coord c;
  c.b = id / per_b;
  int r = id - c.b * per_b;
  const int GMg = 4;
  const int group_sz = GMg * tiles_n;
  const int grp = r / group_sz;
  const int first_m = grp * GMg;
  const int rows_in = min(GMg, tiles_m - first_m);
  r -= grp * group_sz;
  c.tm = first_m + r % rows_in;
  c.tn = r / rows_in;
  return c;
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(WM * WN * 64) gemm_mfma_kernel(const pt_gemm_args g, int tiles_m, int tiles_n) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int A_CH = BM * 8 / NT, B_CH = BN * 8 / NT;  // 16-byte chunks per thread and K step
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = (bf16_t*)smem;            // [2][BM][64]
  bf16_t* Bs = As + 2 * BM * GM_BK;      // [2][BN][64]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const tile_coord tc = map_tile(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  const int m0 = tc.tm * BM, n0 = tc.tn * BN, b = tc.b;

  const bf16_t* A = (const bf16_t*)g.A + b * g.a_bstride;
  const bf16_t* W = (const bf16_t*)g.W + b * g.w_bstride;

  // global -> register staging: chunk id = tid + i*NT; row = id/8, 16-byte chunk = id%8
  const int ld_row = tid >> 3, ld_ch = tid & 7;
  const bf16_t* a_src[A_CH];
  const bf16_t* w_src[B_CH];
  int a_dst[A_CH], w_dst[B_CH];
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int row = ld_row + i * (NT / 8);
    const int gr = min(m0 + row, g.M - 1);
    a_src[i] = A + (int64_t)gr * g.lda + ld_ch * 8;
    a_dst[i] = row * GM_BK + ((ld_ch ^ GM_SWZ(row)) * 8);
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int row = ld_row + i * (NT / 8);
    const int gr = min(n0 + row, g.N - 1);
    w_src[i] = W + (int64_t)gr * g.ldb + ld_ch * 8;
    w_dst[i] = row * GM_BK + ((ld_ch ^ GM_SWZ(row)) * 8);
  }
  u32x4_t a_reg[A_CH], w_reg[B_CH];

  // operand reads: row = tile row + lane%32, chunk = 2*kk + lane/32, swizzled by row%8 = lane%8
  const int fr_row = lane & 31, fr_half = lane >> 5, fr_sw = GM_SWZ(lane & 31);
  int a_off[MI], b_off[NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) a_off[mi] = (wm * TM + mi * 32 + fr_row) * GM_BK;
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) b_off[ni] = (wn * TN + ni * 32 + fr_row) * GM_BK;

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  const int KT = g.K / GM_BK;
  // Software pipeline.  While the MFMAs of K step kt run out of LDS buffer kt&1:
  //   - the global loads of step kt+2 are in flight into registers,
  //   - step kt+1 (loaded one iteration earlier) is stored into the other LDS buffer,
  //   - operand fragments are read one 16-wide sub-step ahead of the MFMAs that use them,
  //   - the single barrier of the iteration sits before the last sub-step's MFMAs, so the first
  //     fragments of step kt+1 are fetched in the shadow of those MFMAs.
  // Steps beyond the end re-read the last one; their copies are never multiplied.
#pragma unroll
  for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const u32x4_t*)(a_src[i]);
#pragma unroll
  for (int i = 0; i < B_CH; ++i) w_reg[i] = *(const u32x4_t*)(w_src[i]);
#pragma unroll
  for (int i = 0; i < A_CH; ++i) *(u32x4_t*)(As + a_dst[i]) = a_reg[i];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) *(u32x4_t*)(Bs + w_dst[i]) = w_reg[i];
  {
    const int koff = min(1, KT - 1) * GM_BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_reg[i] = *(const u32x4_t*)(a_src[i] + koff);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) w_reg[i] = *(const u32x4_t*)(w_src[i] + koff);
  }
  __syncthreads();

  bf16x8_t af[2][MI], bfr[2][NI];
  {
    const int ch = ((0 + fr_half) ^ fr_sw) * 8;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) af[0][mi] = *(const bf16x8_t*)(As + a_off[mi] + ch);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = *(const bf16x8_t*)(Bs + b_off[ni] + ch);
  }

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    u32x4_t a_nxt[A_CH], w_nxt[B_CH];
    const int koff = min(kt + 2, KT - 1) * GM_BK;
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_nxt[i] = *(const u32x4_t*)(a_src[i] + koff);
#pragma unroll
    for (int i = 0; i < B_CH; ++i) w_nxt[i] = *(const u32x4_t*)(w_src[i] + koff);
    __builtin_amdgcn_sched_barrier(0);
    const bf16_t* Ac = As + cur * BM * GM_BK;
    const bf16_t* Bc = Bs + cur * BN * GM_BK;
    bf16_t* An = As + (cur ^ 1) * BM * GM_BK;
    bf16_t* Bn = Bs + (cur ^ 1) * BN * GM_BK;
#pragma unroll
    for (int kk = 0; kk < GM_BK / 16; ++kk) {
      if (kk + 1 < GM_BK / 16) {
        const int ch = (((kk + 1) * 2 + fr_half) ^ fr_sw) * 8;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) af[(kk + 1) & 1][mi] = *(const bf16x8_t*)(Ac + a_off[mi] + ch);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bfr[(kk + 1) & 1][ni] = *(const bf16x8_t*)(Bc + b_off[ni] + ch);
      } else {
        // every wavefront has finished reading this buffer and storing the next one
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int ch = ((0 + fr_half) ^ fr_sw) * 8;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) af[0][mi] = *(const bf16x8_t*)(An + a_off[mi] + ch);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = *(const bf16x8_t*)(Bn + b_off[ni] + ch);
      }
      if (kk == 0) {
#pragma unroll
        for (int i = 0; i < A_CH; ++i) *(u32x4_t*)(An + a_dst[i]) = a_reg[i];
#pragma unroll
        for (int i = 0; i < B_CH; ++i) *(u32x4_t*)(Bn + w_dst[i]) = w_reg[i];
      }
      // fences for the instruction scheduler: keep the LDS traffic of this sub-step ahead of its MFMAs
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][mi], bfr[kk & 1][ni], acc[mi][ni], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_reg[i] = a_nxt[i];
#pragma unroll
    for (int i = 0; i < B_CH; ++i) w_reg[i] = w_nxt[i];
  }
  __syncthreads();

  // ------------------------------------------------------------------ epilogue
  const int col_l = lane & 31;
  const int row_l = 4 * (lane >> 5);
  const int wave_n = n0 + wn * TN;
  const int wave_m = m0 + wm * TM;

  if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_RESIDUAL) {
    float* out = g.out + b * g.out_bstride;
    const float* res = EPI == EPI_RESIDUAL ? g.res + b * g.res_bstride : nullptr;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = wave_m + mi * 32 + 8 * (v >> 2) + row_l + (v & 3);
        if (m < g.M) {
#pragma unroll
          for (int ni = 0; ni < NI; ++ni) {
            const int n = wave_n + ni * 32 + col_l;
            if (n < g.N) {
              const int64_t idx = (int64_t)m * g.ldo + n;
              float x = acc[mi][ni][v];
              if constexpr (EPI == EPI_RESIDUAL) x += res[idx];
              out[idx] = x;
            }
          }
        }
      }
  } else if constexpr (EPI == EPI_SWIGLU) {
    bf16_t* o = (bf16_t*)g.olp + b * g.olp_bstride;
    const int ldo = g.N >> 1;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int m = wave_m + mi * 32 + 8 * (v >> 2) + row_l + (v & 3);
        if (m < g.M) {
#pragma unroll
          for (int ni = 0; ni < NI; ni += 2) {
            const int j = ((wave_n + ni * 32) >> 1) + col_l;   // (phys/64)*32 + lane column
            if (2 * j < g.N) o[(int64_t)m * ldo + j] = f32_to_bf16(silu_f(acc[mi][ni][v]) * acc[mi][ni + 1][v]);
          }
        }
      }
  } else {  // EPI_QKV
    const int hd = g.hd, half = hd >> 1, hq = g.H * hd, hk = g.Hkv * hd;
    const int pstep = hd >> 6;   // partner tile distance: (hd/2)/32
    const bool s4 = (g.S & 3) == 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int mb = wave_m + mi * 32 + 8 * vg + row_l;   // 4 consecutive rows mb..mb+3
        int seq4 = 0, pos4 = 0;
        if (s4) {
          seq4 = mb / g.S;
          pos4 = g.pos0 + (mb - seq4 * g.S);
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int nb = wave_n + ni * 32;   // first column of this 32-wide tile
          if (nb >= g.N) continue;
          if (nb < hq + hk) {
            const bool is_q = nb < hq;
            const int c = is_q ? nb : nb - hq;
            const int head = c / hd, jb = c - head * hd;
            if (jb >= half) continue;   // written together with its low-half partner
            const int j = jb + col_l;
            if (ni + pstep < NI) {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int m = mb + r;
                if (m >= g.M) break;
                int seq, pos;
                if (s4) { seq = seq4; pos = pos4 + r; }
                else { seq = m / g.S; pos = g.pos0 + (m - seq * g.S); }
                const float2 cs = ((const float2*)g.rope)[(int64_t)pos * half + j];
                const float lo = acc[mi][ni][vg * 4 + r];
                const float hi = pstep == 1 ? acc[mi][ni + 1 < NI ? ni + 1 : ni][vg * 4 + r]
                                            : acc[mi][ni + 2 < NI ? ni + 2 : ni][vg * 4 + r];
                const bf16_t rlo = f32_to_bf16(lo * cs.x - hi * cs.y);
                const bf16_t rhi = f32_to_bf16(hi * cs.x + lo * cs.y);
                if (is_q) {
                  bf16_t* q = (bf16_t*)g.olp + b * g.olp_bstride + (int64_t)m * hq + nb + col_l;
                  q[0] = rlo;
                  q[half] = rhi;
                } else {
                  const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
                  bf16_t* k = (bf16_t*)g.kc + hidx * g.kv_head_elems + (int64_t)pos * hd + j;
                  k[0] = rlo;
                  k[half] = rhi;
                }
              }
            }
          } else {
            const int c = nb - hq - hk;
            const int head = c / hd, j = c - head * hd + col_l;
            if (s4 && mb + 3 < g.M) {
              const int64_t hidx = b * g.kv_bstride + seq4 * g.kv_seq_stride + head;
              bf16_t* v = (bf16_t*)g.vc + hidx * ((int64_t)hd * g.s_pad) + (int64_t)j * g.s_pad + pos4;
              uint2 pk;
              pk.x = pack_bf16x2(acc[mi][ni][vg * 4 + 0], acc[mi][ni][vg * 4 + 1]);
              pk.y = pack_bf16x2(acc[mi][ni][vg * 4 + 2], acc[mi][ni][vg * 4 + 3]);
              if ((pos4 & 3) == 0) {
                *(uint2*)v = pk;
              } else {
                v[0] = (bf16_t)(pk.x & 0xffff); v[1] = (bf16_t)(pk.x >> 16);
                v[2] = (bf16_t)(pk.y & 0xffff); v[3] = (bf16_t)(pk.y >> 16);
              }
            } else {
#pragma unroll
              for (int r = 0; r < 4; ++r) {
                const int m = mb + r;
                if (m >= g.M) break;
                const int seq = m / g.S, pos = g.pos0 + (m - seq * g.S);
                const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
                ((bf16_t*)g.vc)[hidx * ((int64_t)hd * g.s_pad) + (int64_t)j * g.s_pad + pos] = f32_to_bf16(acc[mi][ni][vg * 4 + r]);
              }
            }
          }
        }
      }
  }
}

template <int BM, int BN, int WM, int WN, int EPI>
static int launch_cfg(const pt_gemm_args& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (BM + BN) * GM_BK * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, EPI>;
  static bool attr_set = false;
  if (!attr_set) {
    PT_HIP_CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    attr_set = true;
  }
  const int64_t total = (int64_t)tiles_m * tiles_n * g.batch;
  if (total > 0x7fffffff) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "GEMM grid too large");
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(WM * WN * 64), lds, s, g, tiles_m, tiles_n);
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

template <int EPI>
static int launch_epi(const pt_gemm_args& g, hipStream_t s, int cfg) {
  switch (cfg) {
    case 0: return launch_cfg<256, 256, 2, 2, EPI>(g, s);
    case 1: return launch_cfg<256, 256, 4, 2, EPI>(g, s);
    case 2: return launch_cfg<128, 128, 2, 2, EPI>(g, s);
    case 3: return launch_cfg<64, 256, 1, 4, EPI>(g, s);
    case 4: return launch_cfg<128, 256, 2, 2, EPI>(g, s);
    case 5: return launch_cfg<32, 256, 1, 4, EPI>(g, s);
    case 6: return launch_cfg<64, 256, 1, 2, EPI>(g, s);
    default: return launch_cfg<32, 256, 1, 2, EPI>(g, s);
  }
}

// Tile configuration override for tuning runs: -1 = choose by shape.
int pt_gemm_mfma_force_cfg = -1;

#define GM_NCFG 8
static const int kWaveN[GM_NCFG] = {128, 128, 64, 64, 128, 64, 128, 128};   // columns per wavefront

static bool cfg_fits(const pt_gemm_args& g, int cfg) {
  const int wn = kWaveN[cfg];
  if (g.epi == EPI_SWIGLU) return g.N % 64 == 0 && wn % 64 == 0;
  if (g.epi == EPI_QKV) {
    // every wavefront owns whole heads; the q / k / v sections start on wavefront borders
    if (g.hd != 64 && g.hd != 128) return false;
    return wn % g.hd == 0 && (g.H * g.hd) % wn == 0 && (g.Hkv * g.hd) % wn == 0;
  }
  return true;
}

int pt_launch_gemm_mfma(const pt_gemm_args& g, hipStream_t s) {
  if (g.dtype != PT_BF16) return 0;
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return 1;
  if (g.K < GM_BK || g.K % GM_BK) return 0;
  if ((g.lda & 7) || (g.ldb & 7) || (g.a_bstride & 7) || (g.w_bstride & 7)) return 0;
  if (((uintptr_t)g.A | (uintptr_t)g.W) & 15) return 0;
  static const int big[] = {0, 4, 2, -1}, mid[] = {4, 2, -1}, m64[] = {3, 6, -1}, m32[] = {5, 7, -1};
  const int* cand;
  if (g.M <= 32) cand = m32;
  else if (g.M <= 64) cand = m64;
  else if (g.M <= 128 || (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch < 200) cand = mid;
  else cand = big;
  int cfg = -1;
  if (pt_gemm_mfma_force_cfg >= 0 && pt_gemm_mfma_force_cfg < GM_NCFG) {
    if (cfg_fits(g, pt_gemm_mfma_force_cfg)) cfg = pt_gemm_mfma_force_cfg;
  } else {
    for (; *cand >= 0; ++cand)
      if (cfg_fits(g, *cand)) { cfg = *cand; break; }
  }
  if (cfg < 0) return 0;
  switch (g.epi) {
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(g, s, cfg);
    case EPI_RESIDUAL: return launch_epi<EPI_RESIDUAL>(g, s, cfg);
    case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(g, s, cfg);
    case EPI_QKV: return launch_epi<EPI_QKV>(g, s, cfg);
  }
  return 0;
}

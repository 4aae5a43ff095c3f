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
#ifndef PT_GEMM_MFMA_IMPL_H_
#define PT_GEMM_MFMA_IMPL_H_
#include <type_traits>

#include "pt_epilogue.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));   // 16-byte staging register

__device__ __forceinline__ float silu_fast(float z) {
  return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

// Sum of x over each group of LANES (16 or 32) consecutive lanes with data-parallel-primitive adds (no LDS
// traffic): a prefix sum by doubling inside every row of 16 lanes, then lane 15's total carried into the
// next row.  The total of a group is valid in its last lane only.
template <int LANES>
__device__ __forceinline__ float group_sum_last_lane(float x) {
  static_assert(LANES == 16 || LANES == 32, "group width");
  auto shr = [](float v, auto CTRL) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), decltype(CTRL)::value, 0xf, 0xf, true));
  };
  x += shr(x, std::integral_constant<int, 0x111>{});   // row_shr:1
  x += shr(x, std::integral_constant<int, 0x112>{});   // row_shr:2
  x += shr(x, std::integral_constant<int, 0x114>{});   // row_shr:4
  x += shr(x, std::integral_constant<int, 0x118>{});   // row_shr:8
  if constexpr (LANES == 32)                            // row_bcast:15 into rows 1 and 3
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x142, 0xa, 0xf, false));
  return x;
}

#define GM_BK 64   // largest K step; K must be a multiple of 2 * GM_BK

template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

struct tile_coord {
  int b, tm, tn;
};

// Workgroup ids are dealt round-robin to the 8 XCDs (XCD = id % 8), each with its own L2; workgroups of one XCD
// start in id order.  map_tile turns a workgroup id into (track, m-tile, n-tile) such that
//  - the 32 tiles an XCD has in flight form a block of 4 m-tiles x 8 n-tiles (column-major walk through groups of
//    4 m-tiles x all n-tiles): every chunk of A is shared by 8 and every chunk of W by 4 of its workgroups;
//  - when a track's tile grid divides evenly over the XCDs, all XCDs work on the same track at the same time,
//    each on its own range of m-tiles (and, for few m-tiles, of n-tiles).  The weight matrix of that track is then the only W in flight on the whole
//    chip: the Infinity Cache holds it, so the re-reads of W by later m-tile groups stay out of HBM (with one track
//    per XCD, eight weight matrices stream at once and every re-read goes to HBM).
__device__ __forceinline__ tile_coord decode_group(int r, int first_m, int tiles_m, int tiles_n) {
  tile_coord c;
  c.b = 0;
  const int GMg = 4;
  const int group_sz = GMg * tiles_n;
  const int grp = r / group_sz;
  const int gm = grp * GMg;
  const int rows_in = min(GMg, tiles_m - gm);
  r -= grp * group_sz;
  c.tm = first_m + gm + r % rows_in;
  c.tn = r / rows_in;
  return c;
}

__device__ __forceinline__ tile_coord map_tile(int id, int total, int tiles_m, int tiles_n) {
  const int per_b = tiles_m * tiles_n;
  tile_coord c;
  // Split of a track's tile grid over the 8 XCDs, xm ranges of m-tiles by 8 / xm ranges of n-tiles: the most ranges
  // of m-tiles that still leave every XCD four m-tiles (a full 4 x 8 block in flight).
  int xm = 0;
#pragma unroll
  for (int t = 8; t >= 1; t >>= 1)
    if (xm == 0 && tiles_m % t == 0 && tiles_m / t >= 4 && tiles_n % (8 / t) == 0) xm = t;
  if (xm > 0) {
    const int xcd = id & 7, j = id >> 3;          // j-th workgroup of this XCD
    const int per_x = per_b >> 3;                  // tiles of one track that this XCD owns
    const int b = j / per_x;
    const int tm_per = tiles_m / xm, tn_per = tiles_n / (8 / xm);
    c = decode_group(j - b * per_x, (xcd % xm) * tm_per, tm_per, tn_per);
    c.tn += (xcd / xm) * tn_per;
    c.b = b;
    return c;
  }
  // contiguous range of logical ids per XCD
  const int lid = (total & 7) == 0 ? (id & 7) * (total >> 3) + (id >> 3) : id;
  const int b = lid / per_b;
  c = decode_group(lid - b * per_b, 0, tiles_m, tiles_n);
  c.b = b;
  return c;
}

// ------------------------------------------------------------------------------------------------
// Fused epilogues on the accumulator layout of 32x32 MFMA tiles (lane l: column l%32; register v: row
// 8*(v/4) + 4*(l/32) + v%4).  `stage` is the wavefront's private LDS patch (STAGE_ELEMS bf16 elements),
// usable once the K loop is over; wave_m / wave_n are the first row / column of the wavefront's tile.
// ------------------------------------------------------------------------------------------------
// `rs`, when given, holds one factor per row of the wavefront's tile (LDS, index = row - wave_m): the folded
// RMSNorm scale that the QKV and SwiGLU epilogues apply to the accumulators of that row.
typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Instrumented build (the tile-clock benchmark only): every wavefront of gemm_mfma_kernel leaves shader-clock
// stamps of its phases in pt_gemm_stamps[(workgroup * 4 + wavefront) * 8 + i]; i = 0 entry, 1 first MFMA, 2 end of
// the K loop, 3 past the barrier, 4 end of the epilogue; 6 and 7 the constant 100 MHz counter at entry and exit.
#ifdef PT_GEMM_STAMPS
__device__ long long* pt_gemm_stamps = nullptr;
#define PT_STAMP(i)                                                                                                    \
  do {                                                                                                                 \
    if ((threadIdx.x & 63) == 0 && pt_gemm_stamps)                                                                     \
      pt_gemm_stamps[((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + (i)] = ((i) >= 6) ? wall_clock64() : clock64(); \
  } while (0)
#else
#define PT_STAMP(i) ((void)0)
#endif

// Element v of an accumulator tile.  Kernels whose accumulators fill the accumulation registers (more than 128 per
// lane) read them with an explicit v_accvgpr_read at the point of use: left to itself, the register allocator moves
// all of them to vector registers at once when the K loop ends, spills what does not fit to scratch memory, and the
// reloads, each waited for on its own, dominate the epilogue.
template <bool FROM_ACC_REGS>
__device__ __forceinline__ float acc_elem(const f32x16_t& tile, int v) {
  if constexpr (FROM_ACC_REGS) {
    float x;
    asm("v_accvgpr_read_b32 %0, %1" : "=v"(x) : "a"(tile[v]));
    return x;
  } else {
    return tile[v];
  }
}

template <int MI, int NI, int EPI, bool STAGED, int STAGE_ELEMS>
__device__ __forceinline__ void gemm_epilogue(const pt_gemm_args& g, f32x16_t (&acc)[MI][NI], bf16_t* stage, int b,
                                              int wave_m, int wave_n, int lane, const float* rs) {
  constexpr int TN = NI * 32;
  constexpr bool AR = MI * NI * 16 > 128;   // accumulators live in the accumulation registers
  const int col_l = lane & 31;
  const int row_l = 4 * (lane >> 5);
  (void)stage;
  // factor of the row that register v of block mi holds
  auto row_scale = [&](int mi, int v) { return rs ? rs[mi * 32 + 8 * (v >> 2) + row_l + (v & 3)] : 1.0f; };
  (void)row_scale;
  // the factors of all 16 registers of block mi at once (four 16-byte LDS reads, issued before the arithmetic
  // that uses them: a read per register, each waited for on the spot, serialises the epilogue)
  auto row_scales = [&](int mi, float (&rsv)[16]) {
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      f32x4_t t = {1.f, 1.f, 1.f, 1.f};
      if (rs) t = *(const f32x4_t*)(rs + mi * 32 + 8 * vg + row_l);
      rsv[4 * vg + 0] = t.x;
      rsv[4 * vg + 1] = t.y;
      rsv[4 * vg + 2] = t.z;
      rsv[4 * vg + 3] = t.w;
    }
  };
  (void)row_scales;
  if constexpr (EPI == EPI_STORE_F32 || EPI == EPI_RESIDUAL) {
    float* out = g.out + b * g.out_bstride;
    const float* res = EPI == EPI_RESIDUAL ? g.res + b * g.res_bstride : nullptr;
    constexpr int FPITCH = TN + 8;   // floats; +8 keeps the two half-waves on disjoint banks
    constexpr int RCH = 32 * FPITCH * 2 <= STAGE_ELEMS ? 32 : 16;   // rows staged at a time
    if constexpr (STAGED && RCH * FPITCH * 2 <= STAGE_ELEMS) {
      // RCH rows at a time through the wavefront's LDS patch: the accumulator layout (a lane owns a
      // column) becomes row pieces of 4 floats, so the residual read-modify-write moves 16 bytes per
      // lane and whole 128-byte lines per row
      float* fst = (float*)stage;
      constexpr int LPR = TN / 4, RPI = 64 / LPR, ITS = RCH / RPI, NCH = MI * (32 / RCH);
      const int c4 = (lane % LPR) * 4, n = wave_n + c4;
      // folded RMSNorm, producer side: bf16(h * gain) and the row's sum of squares over this wavefront's columns
      const bool fold = EPI == EPI_RESIDUAL && g.nf_out != nullptr;
      f32x4_t gain4 = {1.f, 1.f, 1.f, 1.f};
      if (fold && n < g.N) gain4 = *(const f32x4_t*)(g.nf_gain + b * g.nf_gain_bstride + n);
      // The residual rows of a chunk are loaded one whole chunk ahead of their use (a load from the residual
      // stream takes thousands of clocks under load and nothing else in the workgroup can cover it), where the
      // registers are there: kernels whose accumulators sit in the accumulation registers have the vector
      // registers of the K loop's staging free by now.  The others load in batches of 8 rows.
      constexpr bool PIPE = EPI == EPI_RESIDUAL && (AR || MI * NI * 16 + 8 * ITS <= 160);
      constexpr int BATCH = PIPE ? ITS : (ITS < 8 ? ITS : 8);
      // A wavefront whose tile lies inside the matrix (FULL) runs without the per-row bounds tests: they split the
      // code into small blocks, each of which waits for its own LDS read before it stores.
      auto run = [&](auto FULL_, auto FOLD_) {
        constexpr bool FULL = decltype(FULL_)::value, FOLD = decltype(FOLD_)::value;
        const int row_t = lane / LPR;                                         // the lane's row inside an iteration
        const int64_t lane_off = (int64_t)(wave_m + row_t) * g.ldo + n;     // element offset of the lane's first piece
        f32x4_t rbuf[PIPE ? 2 : 1][BATCH];
        (void)rbuf;
        auto load_res = [&](auto C_, auto IT0_, f32x4_t (&dst)[BATCH]) {
          constexpr int mi = decltype(C_)::value / (32 / RCH), row0 = (decltype(C_)::value % (32 / RCH)) * RCH;
          constexpr int it0 = decltype(IT0_)::value;
          static_for<BATCH>([&](auto I_) {
            constexpr int i = decltype(I_)::value;
            constexpr int r = mi * 32 + row0 + (it0 + i) * RPI;           // row of the iteration inside the tile
            dst[i] = (FULL || (wave_m + r + row_t < g.M && n < g.N)) ? *(const f32x4_t*)(res + lane_off + (int64_t)r * g.ldo)
                                                                     : f32x4_t{0.f, 0.f, 0.f, 0.f};
          });
        };
        if constexpr (PIPE) load_res(std::integral_constant<int, 0>{}, std::integral_constant<int, 0>{}, rbuf[0]);
        static_for<NCH>([&](auto C_) {
          constexpr int c = decltype(C_)::value;
          constexpr int mi = c / (32 / RCH), rc = c % (32 / RCH);
          constexpr int row0 = rc * RCH;                 // first row of the chunk inside the 32-row block
          if constexpr (PIPE && c + 1 < NCH) load_res(std::integral_constant<int, c + 1>{}, std::integral_constant<int, 0>{}, rbuf[(c + 1) & 1]);
          static_for<RCH / 2>([&](auto V_) {
            constexpr int v = (row0 / 8) * 4 + decltype(V_)::value;     // registers whose rows lie in the chunk
            const int row_in = 8 * (v >> 2) + row_l + (v & 3) - row0;
            static_for<NI>([&](auto NI_) {
              constexpr int ni = decltype(NI_)::value;
              fst[row_in * FPITCH + ni * 32 + col_l] = acc_elem<AR>(acc[mi][ni], v);
            });
          });
          static_for<ITS / BATCH>([&](auto B_) {
            constexpr int it0 = decltype(B_)::value * BATCH;
            f32x4_t (&r4)[BATCH] = rbuf[PIPE ? (c & 1) : 0];
            if constexpr (EPI == EPI_RESIDUAL && !PIPE) load_res(C_, std::integral_constant<int, it0>{}, r4);
            f32x4_t x[BATCH];
            float ssv[FOLD ? BATCH : 1];
            (void)ssv;
            static_for<BATCH>([&](auto I_) {
              constexpr int i = decltype(I_)::value;
              x[i] = *(const f32x4_t*)(fst + ((it0 + i) * RPI + row_t) * FPITCH + c4);
            });
            static_for<BATCH>([&](auto I_) {
              constexpr int i = decltype(I_)::value;
              constexpr int r = mi * 32 + row0 + (it0 + i) * RPI;
              const int m = wave_m + r + row_t;
              const bool ok_m = FULL || m < g.M, ok_n = FULL || n < g.N;
              if constexpr (EPI == EPI_RESIDUAL) x[i] += r4[i];
              if (ok_m && ok_n) *(f32x4_t*)(out + lane_off + (int64_t)r * g.ldo) = x[i];
              if constexpr (FOLD) {
                const float ss = ok_n ? x[i].x * x[i].x + x[i].y * x[i].y + x[i].z * x[i].z + x[i].w * x[i].w : 0.f;
                ssv[i] = group_sum_last_lane<LPR>(ss);
                if (ok_m && ok_n) {
                  uint2 pk;
                  pk.x = pack_bf16x2(x[i].x * gain4.x, x[i].y * gain4.y);
                  pk.y = pack_bf16x2(x[i].z * gain4.z, x[i].w * gain4.w);
                  *(uint2*)((bf16_t*)g.nf_out + b * g.nf_out_bstride + (int64_t)m * g.N + n) = pk;
                }
              }
            });
            // the rows' sums of squares, from the last lane of every row group: one divergent branch per batch
            if constexpr (FOLD) {
              if (lane % LPR == LPR - 1) {
                float* ssp = g.nf_ss + b * g.nf_ss_bstride + (int64_t)(wave_m + row_t) * g.nf_parts + wave_n / TN;
                static_for<BATCH>([&](auto I_) {
                  constexpr int i = decltype(I_)::value;
                  constexpr int r = mi * 32 + row0 + (it0 + i) * RPI;
                  if (FULL || wave_m + r + row_t < g.M) ssp[(int64_t)r * g.nf_parts] = ssv[i];
                });
              }
            }
          });
        });
      };
      const bool full = wave_m + MI * 32 <= g.M && wave_n + TN <= g.N;
      if constexpr (EPI == EPI_RESIDUAL) {
        if (fold) { if (full) run(std::true_type{}, std::true_type{}); else run(std::false_type{}, std::true_type{}); }
        else { if (full) run(std::true_type{}, std::false_type{}); else run(std::false_type{}, std::false_type{}); }
      } else {
        if (full) run(std::true_type{}, std::false_type{}); else run(std::false_type{}, std::false_type{});
      }
    } else {
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
                float x = acc_elem<AR>(acc[mi][ni], v);
                if constexpr (EPI == EPI_RESIDUAL) x += res[idx];
                out[idx] = x;
              }
            }
          }
        }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
    bf16_t* o = (bf16_t*)g.olp + b * g.olp_bstride;
    const int ldo = g.N >> 1;
    if constexpr (STAGED) {
      // 32 rows at a time: products go to the wavefront's LDS patch as bf16, come back as 16-byte
      // row pieces and leave as full 128-byte lines
      constexpr int OC = TN / 2, PITCH = OC + 8, LPR = OC / 8, RPI = 64 / LPR;
      static_assert(32 * PITCH <= STAGE_ELEMS, "staging patch too small");
      const bool full = wave_m + MI * 32 <= g.M && wave_n + TN <= g.N;
      static_for<MI>([&](auto MI_) {
        constexpr int mi = decltype(MI_)::value;
        float rsv[16];
        row_scales(mi, rsv);
        static_for<16>([&](auto V_) {
          constexpr int v = decltype(V_)::value;
          const int row_in = 8 * (v >> 2) + row_l + (v & 3);
          const float rsc = rsv[v];
          static_for<NI / 2>([&](auto P_) {
            constexpr int pp = decltype(P_)::value;
            stage[row_in * PITCH + 32 * pp + col_l] = f32_to_bf16(silu_fast(rsc * acc_elem<AR>(acc[mi][2 * pp], v)) * (rsc * acc_elem<AR>(acc[mi][2 * pp + 1], v)));
          });
          if constexpr ((v & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // bounds the scheduler's window (register pressure)
        });
        // a wavefront whose tile lies inside the matrix stores without bounds tests, all LDS reads first
        const int row_t = lane / LPR, chunk = lane % LPR;
        const int j = (wave_n >> 1) + chunk * 8;
        const bf16_t* src = stage + row_t * PITCH + chunk * 8;
        bf16_t* dst = o + (int64_t)(wave_m + mi * 32 + row_t) * ldo + j;
        u32x4_t val[32 / RPI];
        static_for<32 / RPI>([&](auto IT_) {
          constexpr int it = decltype(IT_)::value;
          val[it] = *(const u32x4_t*)(src + it * RPI * PITCH);
        });
        if (full) {
          static_for<32 / RPI>([&](auto IT_) {
            constexpr int it = decltype(IT_)::value;
            *(u32x4_t*)(dst + (int64_t)(it * RPI) * ldo) = val[it];
          });
        } else {
          static_for<32 / RPI>([&](auto IT_) {
            constexpr int it = decltype(IT_)::value;
            if (wave_m + mi * 32 + it * RPI + row_t < g.M && 2 * j < g.N) *(u32x4_t*)(dst + (int64_t)(it * RPI) * ldo) = val[it];
          });
        }
      });
    } else {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int m = wave_m + mi * 32 + 8 * (v >> 2) + row_l + (v & 3);
          if (m < g.M) {
#pragma unroll
            for (int ni = 0; ni < NI; ni += 2) {
              const int j = ((wave_n + ni * 32) >> 1) + col_l;   // (phys/64)*32 + lane column
              const float rsc = row_scale(mi, v);
              if (2 * j < g.N) o[(int64_t)m * ldo + j] = f32_to_bf16(silu_fast(rsc * acc_elem<AR>(acc[mi][ni], v)) * (rsc * acc_elem<AR>(acc[mi][ni + 1], v)));
            }
          }
        }
    }
  } else {  // EPI_QKV
    const int hd = g.hd, half = hd >> 1, hq = g.H * hd, hk = g.Hkv * hd;
    const bool wide = hd == 128;     // partner tile distance (hd/2)/32: 1 for hd 64, 2 for hd 128
    const int hd_sh = wide ? 7 : 6;  // hd is 64 or 128 here: shifts and masks instead of runtime divisions
    // 4 consecutive rows of a register group lie in one sequence, at consecutive positions
    const bool s4 = g.row_map ? g.row_blocks != 0 : (g.S & 3) == 0;
    constexpr int QPITCH = TN + 8;   // bf16 elements per staged row of q / k
    constexpr int VPITCH = 32 + 8;   // bf16 elements per staged V^T row (32 positions)
    constexpr bool CAN_STAGE = STAGED && 32 * QPITCH <= STAGE_ELEMS && TN * VPITCH <= STAGE_ELEMS;
    bool staged_done = false;
    if constexpr (CAN_STAGE) {
      // Aligned prefill (32-row blocks inside one sequence, positions a multiple of 8): 32 rows at a
      // time go through the wavefront's LDS patch.  q and k are rotated in registers, staged row-major
      // and leave as 16-byte row pieces; v is staged transposed and leaves as 16-byte pieces of V^T
      // rows (8 consecutive positions of one head-dim index).
      if ((g.row_map ? g.row_blocks != 0 : (g.S & 31) == 0) && (g.pos0 & 7) == 0 && wave_n < g.N) {
        staged_done = true;
        const bool is_qk = wave_n < hq + hk, is_q = wave_n < hq;
        // The head width as a constant: a wavefront owns whole heads (wave_n is a multiple of hd), so which
        // 32-column tiles hold the low halves, and where their partners are, is then known at compile time.
        auto staged_part = [&](auto WIDE_) {
          constexpr bool W = decltype(WIDE_)::value;
          constexpr int HD = W ? 128 : 64, HALF = HD / 2, NW = HALF / 32;   // NW low-half tiles per head
          // cos/sin of (position, column): the table is read once per 32-row block, for the lane's first row;
          // the lane's other rows follow by rotating with the table's entries for 1 and 5 positions (its rows
          // are r, r+1, r+2, r+3, r+8, ...).  All loads are issued before the first staging store: a load after
          // a store through the staging pointer would wait for it, and the registers to keep one table entry
          // per accumulator element in flight are not there.  Low-half tile w of a head uses column col_l + 32 w.
          float2 cs_base[MI][NW], rot1[NW], rot5[NW];
          if (is_qk) {
            const float2* tab = (const float2*)g.rope + col_l;
#pragma unroll
            for (int w = 0; w < NW; ++w) {
              rot1[w] = tab[HALF + 32 * w];
              rot5[w] = tab[5 * HALF + 32 * w];
            }
            static_for<MI>([&](auto MI_) {
              constexpr int mi = decltype(MI_)::value;
              const int mrow0 = min(wave_m + mi * 32, g.M - 32);
              const int pos0b = gemm_row_pos(g, mrow0).pos;
              const float2* rp = tab + (int64_t)(pos0b + row_l) * HALF;
#pragma unroll
              for (int w = 0; w < NW; ++w) cs_base[mi][w] = rp[32 * w];
            });
          }
          static_for<MI>([&](auto MI_) {
            constexpr int mi = decltype(MI_)::value;
            const int mrow0 = wave_m + mi * 32;           // first row of the block
            if (mrow0 < g.M) {
              const pt_rowpos rp0 = gemm_row_pos(g, mrow0);
              const int seq = rp0.seq, pos0b = rp0.pos;
              float rsv[16];
              row_scales(mi, rsv);
              if (is_qk) {
                float2 cs_cur[NW];
#pragma unroll
                for (int w = 0; w < NW; ++w) cs_cur[w] = cs_base[mi][w];
                bf16_t* st = stage + row_l * QPITCH + col_l;
                static_for<16>([&](auto V_) {
                  constexpr int v = decltype(V_)::value;
                  constexpr int row_c = 8 * (v >> 2) + (v & 3);   // row inside the block, less row_l
                  const float rsc = rsv[v];
                  if constexpr (v > 0) {
#pragma unroll
                    for (int w = 0; w < NW; ++w) {
                      const float2 r = (v & 3) == 0 ? rot5[w] : rot1[w];
                      const float2 c = cs_cur[w];
                      cs_cur[w].x = c.x * r.x - c.y * r.y;
                      cs_cur[w].y = c.y * r.x + c.x * r.y;
                    }
                  }
                  static_for<NI>([&](auto NI_) {
                    constexpr int ni = decltype(NI_)::value;
                    constexpr int jb = (ni * 32) & (HD - 1);
                    constexpr int pn = ni + NW < NI ? ni + NW : ni;   // the tile with the partner columns
                    if constexpr (jb < HALF) {
                      const float2 cs = cs_cur[jb / 32];
                      const float lo = rsc * acc_elem<AR>(acc[mi][ni], v);
                      const float hi = rsc * acc_elem<AR>(acc[mi][pn], v);
                      st[row_c * QPITCH + ni * 32] = f32_to_bf16(lo * cs.x - hi * cs.y);
                      st[row_c * QPITCH + ni * 32 + HALF] = f32_to_bf16(hi * cs.x + lo * cs.y);
                    }
                  });
                });
                constexpr int LPR = TN / 8, RPI = 64 / LPR;
                const int c8 = (lane % LPR) * 8;
                const int c = (is_q ? wave_n : wave_n - hq) + c8;       // column inside the q or k section
                const int head = c / HD, j = c % HD;
                bf16_t* dst = is_q ? (bf16_t*)g.olp + b * g.olp_bstride + (int64_t)(mrow0 + lane / LPR) * hq + c
                                   : (bf16_t*)g.kc + (b * g.kv_bstride + seq * g.kv_seq_stride + head) * g.kv_head_elems +
                                         (int64_t)(pos0b + lane / LPR) * HD + j;
                const int64_t dpitch = is_q ? hq : HD;                  // elements per row at the destination
                const bf16_t* src = stage + (lane / LPR) * QPITCH + c8;
                static_for<32 / RPI>([&](auto IT_) {
                  constexpr int it = decltype(IT_)::value;
                  *(u32x4_t*)(dst + it * RPI * dpitch) = *(const u32x4_t*)(src + it * RPI * QPITCH);
                });
              } else {
                static_for<4>([&](auto VG_) {
                  constexpr int vg = decltype(VG_)::value;
                  static_for<NI>([&](auto NI_) {
                    constexpr int ni = decltype(NI_)::value;
                    uint2 pk;
                    pk.x = pack_bf16x2(rsv[vg * 4 + 0] * acc_elem<AR>(acc[mi][ni], vg * 4 + 0), rsv[vg * 4 + 1] * acc_elem<AR>(acc[mi][ni], vg * 4 + 1));
                    pk.y = pack_bf16x2(rsv[vg * 4 + 2] * acc_elem<AR>(acc[mi][ni], vg * 4 + 2), rsv[vg * 4 + 3] * acc_elem<AR>(acc[mi][ni], vg * 4 + 3));
                    *(uint2*)(stage + (ni * 32 + col_l) * VPITCH + 8 * vg + row_l) = pk;
                  });
                });
                const int p8 = (lane & 3) * 8;
                // a wavefront's columns lie in whole heads: head and head-dim index of column (lane >> 2)
                const int c0 = wave_n - hq - hk + (lane >> 2);
                const int head0 = c0 / HD, j0 = c0 % HD;
                bf16_t* dst = (bf16_t*)g.vc + (b * g.kv_bstride + seq * g.kv_seq_stride + head0) * ((int64_t)HD * g.s_pad) +
                              (int64_t)j0 * g.s_pad + pos0b + p8;
                const bf16_t* src = stage + (lane >> 2) * VPITCH + p8;
                static_for<TN / 16>([&](auto IT_) {
                  constexpr int it = decltype(IT_)::value;
                  // column it*16 further on: the head-dim rows of V^T are s_pad apart and heads follow one another
                  *(u32x4_t*)(dst + (int64_t)(it * 16) * g.s_pad) = *(const u32x4_t*)(src + it * 16 * VPITCH);
                });
              }
            }
          });
        };
        if (wide) staged_part(std::true_type{});
        else staged_part(std::false_type{});
      }
    }
    if (!staged_done)
    static_for<MI>([&](auto MI_) {
      constexpr int mi = decltype(MI_)::value;
      static_for<4>([&](auto VG_) {
        constexpr int vg = decltype(VG_)::value;
        const int mb = wave_m + mi * 32 + 8 * vg + row_l;   // rows mb .. mb+3
        int seq4 = 0, pos4 = 0;
        if (s4) {
          const pt_rowpos rp4 = gemm_row_pos(g, min(mb, g.M - 1));
          seq4 = rp4.seq;
          pos4 = rp4.pos;
        }
        static_for<NI>([&](auto NI_) {
          constexpr int ni = decltype(NI_)::value;
          const int nb = wave_n + ni * 32;   // first column of this 32-wide tile (wave-uniform)
          if (nb < hq + hk) {
            // q or k: rotate (u_j, u_{j+hd/2}); the low half owns the pair
            const bool is_q = nb < hq;
            const int c = is_q ? nb : nb - hq;
            const int head = c >> hd_sh, jb = c & (hd - 1);
            if (jb < half && nb < g.N) {
              const int j = jb + col_l;
              constexpr int p1 = ni + 1 < NI ? ni + 1 : ni, p2 = ni + 2 < NI ? ni + 2 : ni;
              static_for<4>([&](auto R_) {
                constexpr int r = decltype(R_)::value;
                const int m = mb + r;
                if (m < g.M) {
                  int seq, pos;
                  if (s4) { seq = seq4; pos = pos4 + r; }
                  else { const pt_rowpos rpm = gemm_row_pos(g, m); seq = rpm.seq; pos = rpm.pos; }
                  const float2 cs = ((const float2*)g.rope)[(int64_t)pos * half + j];
                  const float rsc = row_scale(mi, vg * 4 + r);
                  const float lo = rsc * acc_elem<AR>(acc[mi][ni], vg * 4 + r);
                  const float hi = rsc * (wide ? acc_elem<AR>(acc[mi][p2], vg * 4 + r) : acc_elem<AR>(acc[mi][p1], vg * 4 + r));
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
              });
            }
          } else if (nb < g.N) {
            // v: transposed store, 4 consecutive positions of one head-dim row
            const int c = nb - hq - hk;
            const int head = c >> hd_sh, j = (c & (hd - 1)) + col_l;
            if (s4 && mb + 3 < g.M && (pos4 & 3) == 0) {
              const int64_t hidx = b * g.kv_bstride + seq4 * g.kv_seq_stride + head;
              bf16_t* v = (bf16_t*)g.vc + hidx * ((int64_t)hd * g.s_pad) + (int64_t)j * g.s_pad + pos4;
              uint2 pk;
              pk.x = pack_bf16x2(row_scale(mi, vg * 4 + 0) * acc_elem<AR>(acc[mi][ni], vg * 4 + 0), row_scale(mi, vg * 4 + 1) * acc_elem<AR>(acc[mi][ni], vg * 4 + 1));
              pk.y = pack_bf16x2(row_scale(mi, vg * 4 + 2) * acc_elem<AR>(acc[mi][ni], vg * 4 + 2), row_scale(mi, vg * 4 + 3) * acc_elem<AR>(acc[mi][ni], vg * 4 + 3));
              *(uint2*)v = pk;
            } else {
              static_for<4>([&](auto R_) {
                constexpr int r = decltype(R_)::value;
                const int m = mb + r;
                if (m < g.M) {
                  const pt_rowpos rpm = gemm_row_pos(g, m);
                  const int seq = rpm.seq, pos = rpm.pos;
                  const int64_t hidx = b * g.kv_bstride + seq * g.kv_seq_stride + head;
                  ((bf16_t*)g.vc)[hidx * ((int64_t)hd * g.s_pad) + (int64_t)j * g.s_pad + pos] = f32_to_bf16(row_scale(mi, vg * 4 + r) * acc_elem<AR>(acc[mi][ni], vg * 4 + r));
                }
              });
            }
          }
        });
      });
    });
  }
}

template <int BM, int BN, int WM, int WN, int BK, int EPI>
__global__ void __launch_bounds__(WM * WN * 64, (2 * (BM + BN) * BK * 2 <= 80 * 1024 && BM * BN <= 256 * 128 && WM * WN == 4) ? 2 : 1)
gemm_mfma_kernel(const pt_gemm_args g, int tiles_m, int tiles_n) {
  PT_STAMP(6);
  PT_STAMP(0);
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int CPR = BK / 8;        // 16-byte chunks per LDS row
  constexpr int SS = BK / 16;        // MFMA sub-steps per K step
  constexpr int A_CH = BM * CPR / NT, B_CH = BN * CPR / NT;  // 16-byte chunks per thread and K step
  static_assert(BK == 64 || BK == 32, "K step");
  static_assert(BM * CPR % NT == 0 && BN * CPR % NT == 0, "tile/threads mismatch");
  // XOR swizzle of the 16-byte chunks: any 16 consecutive rows reading the same logical chunk hit 16
  // different 16-byte columns of a 256-byte LDS line (gfx950 serves 16 lanes x 16 B per clock)
  auto SWZ = [](int row) { return BK == 64 ? ((row >> 1) & 7) : ((row >> 2) & 3); };
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* As = (bf16_t*)smem;            // [2][BM][BK]
  bf16_t* Bs = As + 2 * BM * BK;      // [2][BN][BK]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const tile_coord tc = map_tile(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  // the tile's coordinates are the same for every lane: kept in scalar registers (the divisions of the tile walk
  // leave them in vector registers, where their 64-bit products crowd the K loop and get spilled around it)
  const int m0 = __builtin_amdgcn_readfirstlane(tc.tm) * BM, n0 = __builtin_amdgcn_readfirstlane(tc.tn) * BN,
            b = __builtin_amdgcn_readfirstlane(tc.b);
  // grouped GEMM: the weight matrix of this tile's rows; tiles that start in a block without rows have nothing to do
  int group = 0;
  if (g.blk_group) {
    group = g.blk_group[b * g.grp_bstride + (m0 >> 6)];
    if (group < 0) return;
  }

  // folded RMSNorm, consumer side: one factor per tile row (1/rms of the row, from pt_launch_row_inv_rms).  The
  // load is issued here and parked in LDS only after the K loop, so nothing waits for it.
  __shared__ __attribute__((aligned(16))) float rs_inv[BM];
  const bool has_rs = (EPI == EPI_QKV || EPI == EPI_SWIGLU) && g.rs_inv != nullptr;
  static_assert(BM <= NT, "one factor per thread");
  float rs_mine = 1.0f;
  if (has_rs) rs_mine = g.rs_inv[b * g.rs_bstride + min(m0 + min(tid, BM - 1), g.M - 1)];   // wave-uniform branch

  // global -> register staging: chunk id = tid + i*NT; row = id/CPR, 16-byte chunk = id%CPR.
  // Rows of one thread are NT/CPR apart, a multiple of 16, so they share the swizzle and the LDS
  // destinations differ by a constant.
  const int ld_row = tid / CPR, ld_ch = tid % CPR;
  static_assert((NT / CPR) % 16 == 0, "staging rows must keep the swizzle");
  constexpr int ST_STRIDE = (NT / CPR) * BK;                    // elements between a thread's staging rows
  const int st_dst = ld_row * BK + ((ld_ch ^ SWZ(ld_row)) * 8);
  u32x4_t a_reg[2][A_CH], w_reg[2][B_CH];                        // two staging sets: K steps of equal parity

  const int KT = g.K / BK;   // even, >= 2
  uint32_t a_voff[A_CH], w_voff[B_CH];   // byte offsets from the tile's first row
#pragma unroll
  for (int i = 0; i < A_CH; ++i) {
    const int m = min(m0 + ld_row + i * (NT / CPR), g.M - 1);
    // gathered rows (grouped GEMM) are addressed from the track's first row: the host checks rows * lda * 2 < 2^32
    const uint32_t gr = g.a_rows ? (uint32_t)g.a_rows[b * g.a_rows_bstride + m] : (uint32_t)(m - m0);
    a_voff[i] = (gr * (uint32_t)g.lda + ld_ch * 8) * 2;
  }
#pragma unroll
  for (int i = 0; i < B_CH; ++i) {
    const int gr = min(n0 + ld_row + i * (NT / CPR), g.N - 1) - n0;
    w_voff[i] = (uint32_t)((gr * g.ldb + ld_ch * 8) * 2);
  }
  const char* a_base = (const char*)((const bf16_t*)g.A + b * g.a_bstride + (g.a_rows ? 0 : (int64_t)m0 * g.lda));   // wave-uniform
  const char* w_base = (const char*)((const bf16_t*)g.W + b * g.w_bstride + group * g.w_gstride + (int64_t)n0 * g.ldb);
  auto load_a = [&](int set, int i, int kstep) { a_reg[set][i] = *(const u32x4_t*)(a_base + (size_t)kstep * (BK * 2) + a_voff[i]); };
  auto load_w = [&](int set, int i, int kstep) { w_reg[set][i] = *(const u32x4_t*)(w_base + (size_t)kstep * (BK * 2) + w_voff[i]); };

  // operand reads: row = tile row + lane%32, 16-byte chunk = 2*kk + lane/32, swizzled by the row
  const int fr_row = lane & 31, fr_half = lane >> 5, fr_sw = SWZ(lane & 31);
  int a_fr[SS], b_fr[SS];   // element offsets of sub-step kk inside a buffer, first MFMA tile of the wavefront
#pragma unroll
  for (int kk = 0; kk < SS; ++kk) {
    const int ch = ((kk * 2 + fr_half) ^ fr_sw) * 8;
    a_fr[kk] = (wm * TM + fr_row) * BK + ch;
    b_fr[kk] = (wn * TN + fr_row) * BK + ch;
  }

  // Software pipeline (K step = 64).  In every iteration the MFMAs run out of LDS buffer `cur` while
  //   sub-steps 0..2: the next K step (staging set cur^1, loaded two iterations ago) is stored into the
  //                   other LDS buffer chunk by chunk, and every chunk's register is refilled right away
  //                   from global memory with the K step three ahead: a load has two whole iterations to
  //                   arrive, which matters because about a fifth of them miss the XCD's L2 (measured:
  //                   +2.4 % on model data, +4.8 % on zeros over refilling in sub-steps 2 and 3),
  //   every sub-step: the operand fragments of the next sub-step are read from LDS,
  // and every memory instruction is issued between two MFMAs, so no queue sees a burst.  The one
  // barrier of the iteration sits in front of sub-step 3: after it the first fragments of the next
  // K step are fetched in the shadow of the last MFMAs.
#pragma unroll
  for (int i = 0; i < A_CH; ++i) load_a(0, i, 0);
#pragma unroll
  for (int i = 0; i < B_CH; ++i) load_w(0, i, 0);
#pragma unroll
  for (int i = 0; i < A_CH; ++i) load_a(1, i, 1);
#pragma unroll
  for (int i = 0; i < B_CH; ++i) load_w(1, i, 1);
#pragma unroll
  for (int i = 0; i < A_CH; ++i) *(u32x4_t*)(As + st_dst + i * ST_STRIDE) = a_reg[0][i];
#pragma unroll
  for (int i = 0; i < B_CH; ++i) *(u32x4_t*)(Bs + st_dst + i * ST_STRIDE) = w_reg[0][i];
  // The largest tile leaves the loads of K step 2 to its first iteration, between the MFMAs.
  constexpr bool LATE2 = BM * BN >= 256 * 256;
  if constexpr (!LATE2) {
#pragma unroll
    for (int i = 0; i < A_CH; ++i) load_a(0, i, min(2, KT - 1));
#pragma unroll
    for (int i = 0; i < B_CH; ++i) load_w(0, i, min(2, KT - 1));
  }
  __syncthreads();
  bf16x8_t af[2][MI], bfr[2][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) af[0][mi] = *(const bf16x8_t*)(As + a_fr[0] + mi * 32 * BK);
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = *(const bf16x8_t*)(Bs + b_fr[0] + ni * 32 * BK);

  constexpr int NM = MI * NI;                  // MFMAs per sub-step
  constexpr int FR = MI + NI;                  // fragment reads per sub-step
  constexpr int EX = A_CH + B_CH;              // staging chunks per K step
  constexpr int NS = SS - 1;                   // sub-steps in front of the barrier: each parks its share of the staging chunks and refills them
  constexpr int EXS = (EX + NS - 1) / NS;      // staging chunks handled per such sub-step

  f32x16_t acc[MI][NI];

  // FIRST: the iteration of K step 0, which also loads K step 2 into the staging set that the pipeline fill has
  // just parked (a wavefront can keep 63 loads in flight: issued in front of the loop, those loads would hold
  // the first MFMA back until the loads of K step 1 have returned).
  auto iteration = [&](auto PAR, auto FIRST_, int kt) {
    constexpr int cur = decltype(PAR)::value;          // LDS buffer being multiplied
    constexpr bool FIRST = decltype(FIRST_)::value;
    constexpr int PER = FIRST ? 3 : 2;                  // memory instructions per staging chunk
    constexpr int wset = cur ^ 1;                       // staging set stored, then reloaded
    const bf16_t* Ac = As + cur * BM * BK;
    const bf16_t* Bc = Bs + cur * BN * BK;
    bf16_t* An = As + (cur ^ 1) * BM * BK;
    bf16_t* Bn = Bs + (cur ^ 1) * BN * BK;
    const int kload = min(kt + 3, KT - 1);   // K steps past the end re-read the last one (never multiplied)
    static_for<SS>([&](auto KK) {
      constexpr int kk = decltype(KK)::value;
      constexpr int fb = (kk + 1) & 1;                  // fragment buffer being filled
      constexpr int R = kk < NS ? FR + PER * EXS : FR;   // memory instructions of this sub-step
      if constexpr (kk == SS - 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
      static_for<NM>([&](auto J) {
        constexpr int j = decltype(J)::value;
        constexpr int mi = j / NI, ni = j % NI;
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][mi], bfr[kk & 1][ni], acc[mi][ni], 0, 0, 0);
        constexpr int lo = j * R / NM, hi = (j + 1) * R / NM;
        static_for<hi - lo>([&](auto RR) {
          constexpr int r = lo + decltype(RR)::value;
          if constexpr (r < MI) {
            const bf16_t* src = kk == SS - 1 ? An + a_fr[0] : Ac + a_fr[(kk + 1) % SS];
            af[fb][r] = *(const bf16x8_t*)(src + r * 32 * BK);
          } else if constexpr (r < FR) {
            const bf16_t* src = kk == SS - 1 ? Bn + b_fr[0] : Bc + b_fr[(kk + 1) % SS];
            bfr[fb][r - MI] = *(const bf16x8_t*)(src + (r - MI) * 32 * BK);
          } else {
            constexpr int e = kk * EXS + (r - FR) / PER;   // staging chunk: parked, then refilled right away
            constexpr int what = (r - FR) % PER + (FIRST ? 0 : 1);   // 0: load of K step 2, 1: park, 2: refill
            if constexpr (e < EX && kk < NS) {
              if constexpr (what == 0) {
                if constexpr (e < A_CH) load_a(cur, e, min(2, KT - 1));
                else load_w(cur, e - A_CH, min(2, KT - 1));
              } else if constexpr (what == 1) {
                if constexpr (e < A_CH) *(u32x4_t*)(An + st_dst + e * ST_STRIDE) = a_reg[wset][e];
                else *(u32x4_t*)(Bn + st_dst + (e - A_CH) * ST_STRIDE) = w_reg[wset][e - A_CH];
              } else {
                if constexpr (e < A_CH) load_a(wset, e, kload);
                else load_w(wset, e - A_CH, kload);
              }
            }
          }
        });
        __builtin_amdgcn_sched_barrier(0);
      });
    });
  };

#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
  PT_STAMP(1);
  if constexpr (LATE2) {
    iteration(std::integral_constant<int, 0>{}, std::true_type{}, 0);
    iteration(std::integral_constant<int, 1>{}, std::false_type{}, 1);
  }
  for (int kt = LATE2 ? 2 : 0; kt < KT; kt += 2) {
    iteration(std::integral_constant<int, 0>{}, std::false_type{}, kt);
    iteration(std::integral_constant<int, 1>{}, std::false_type{}, kt + 1);
  }
  PT_STAMP(2);
  if (has_rs && tid < BM) rs_inv[tid] = rs_mine;
  __syncthreads();   // LDS is free for the staged epilogues
  PT_STAMP(3);

  // ------------------------------------------------------------------ epilogue
  // LDS patch of this wavefront for the staged epilogues (the K loop is over: all of LDS is free)
  constexpr bool STAGED = BM >= 128 && BN >= 128;
  constexpr int STAGE_ELEMS = 2 * (BM + BN) * BK / (WM * WN);   // per wavefront
  bf16_t* stage = (bf16_t*)smem + wave * STAGE_ELEMS;
  (void)stage;
  const int wave_n = n0 + wn * TN;
  const int wave_m = m0 + wm * TM;

  gemm_epilogue<MI, NI, EPI, STAGED, STAGE_ELEMS>(g, acc, stage, b, wave_m, wave_n, lane, has_rs ? rs_inv + wm * TM : nullptr);
  PT_STAMP(4);
  PT_STAMP(7);
}

// ------------------------------------------------------------------------------------------------
// Variant with direct global -> LDS loads (gfx950 global_load_lds_dwordx4): operand tiles never touch
// registers on their way in.  K step 32, four LDS stages; the loads of K step kt+3 are issued while
// step kt is multiplied, so three steps are always in flight.  A wavefront instruction moves 64 x 16
// bytes into 1024 consecutive LDS bytes = 16 rows of 64 bytes; lane L therefore fetches, for row L/4,
// the logical chunk (L%4) ^ swizzle(row), which yields the same conflict-free swizzled layout as the
// register-staged kernel.  With 8 wavefronts (2 per SIMD, 128 accumulator registers each) one
// wavefront's LDS and barrier waits are covered by the other's MFMAs.
// ------------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(WM * WN * 64, WM * WN == 8 ? 2 : 1)
gemm_dl_kernel(const pt_gemm_args g, int tiles_m, int tiles_n) {
  constexpr int BK = 32, NSTG = 4, NW = WM * WN;
  constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
  constexpr int STG = (BM + BN) * BK;                 // elements per stage: A rows then W rows
  constexpr int LA = BM / 16 / NW, LB = BN / 16 / NW; // 16-row groups (= load instructions) per wavefront and K step
  static_assert(BM / 16 % NW == 0 && BN / 16 % NW == 0, "tile/wavefront mismatch");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* lds = (bf16_t*)smem;
  auto SWZ = [](int row) { return (row >> 2) & 3; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const tile_coord tc = map_tile(blockIdx.x, gridDim.x, tiles_m, tiles_n);
  // the tile's coordinates are the same for every lane: kept in scalar registers (the divisions of the tile walk
  // leave them in vector registers, where their 64-bit products crowd the K loop and get spilled around it)
  const int m0 = __builtin_amdgcn_readfirstlane(tc.tm) * BM, n0 = __builtin_amdgcn_readfirstlane(tc.tn) * BN,
            b = __builtin_amdgcn_readfirstlane(tc.b);
  const int KT = g.K / BK;   // multiple of 4
  int group = 0;             // grouped GEMM, as in gemm_mfma_kernel
  if (g.blk_group) {
    group = g.blk_group[b * g.grp_bstride + (m0 >> 6)];
    if (group < 0) return;
  }

  // folded RMSNorm, consumer side: one factor per tile row (1/rms of the row, from pt_launch_row_inv_rms).  The
  // load is issued here and parked in LDS only after the K loop, so nothing waits for it.
  __shared__ __attribute__((aligned(16))) float rs_inv[BM];
  const bool has_rs = (EPI == EPI_QKV || EPI == EPI_SWIGLU) && g.rs_inv != nullptr;
  static_assert(BM <= (NW * 64), "one factor per thread");
  float rs_mine = 1.0f;
  if (has_rs) rs_mine = g.rs_inv[b * g.rs_bstride + min(m0 + min(tid, BM - 1), g.M - 1)];   // wave-uniform branch

  // direct loads: group grp covers tile rows grp*16 .. +15; this lane fetches row L/4, logical chunk (L%4)^swz
  const int rr = lane >> 2, pc = lane & 3;
  uint32_t a_voff[LA], w_voff[LB];
#pragma unroll
  for (int i = 0; i < LA; ++i) {
    const int row = (wave * LA + i) * 16 + rr;
    const int m = min(m0 + row, g.M - 1);
    const uint32_t gr = g.a_rows ? (uint32_t)g.a_rows[b * g.a_rows_bstride + m] : (uint32_t)(m - m0);
    a_voff[i] = (gr * (uint32_t)g.lda + (pc ^ SWZ(row)) * 8) * 2;
  }
#pragma unroll
  for (int i = 0; i < LB; ++i) {
    const int row = (wave * LB + i) * 16 + rr;
    const int gr = min(n0 + row, g.N - 1) - n0;
    w_voff[i] = (uint32_t)((gr * g.ldb + (pc ^ SWZ(row)) * 8) * 2);
  }
  const char* a_base = (const char*)((const bf16_t*)g.A + b * g.a_bstride + (g.a_rows ? 0 : (int64_t)m0 * g.lda));
  const char* w_base = (const char*)((const bf16_t*)g.W + b * g.w_bstride + group * g.w_gstride + (int64_t)n0 * g.ldb);
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  auto issue_load = [&](int i, int kstep, int stage) {   // i < LA: A group, else W group
    if (i < LA)
      __builtin_amdgcn_global_load_lds((gptr_t)(a_base + (size_t)kstep * (BK * 2) + a_voff[i]),
                                       (lptr_t)(lds + stage * STG + (wave * LA + i) * 16 * BK), 16, 0, 0);
    else
      __builtin_amdgcn_global_load_lds((gptr_t)(w_base + (size_t)kstep * (BK * 2) + w_voff[i - LA]),
                                       (lptr_t)(lds + stage * STG + BM * BK + (wave * LB + (i - LA)) * 16 * BK), 16, 0, 0);
  };

  // operand fragments: row = tile row + lane%32, 16-byte chunk = 2*kk + lane/32, swizzled by the row
  const int fr_row = lane & 31, fr_half = lane >> 5;
  int a_fr[2], b_fr[2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk) {
    const int ra = wm * TM + fr_row, rb = wn * TN + fr_row;
    a_fr[kk] = ra * BK + (((kk * 2 + fr_half) ^ SWZ(ra)) * 8);
    b_fr[kk] = BM * BK + rb * BK + (((kk * 2 + fr_half) ^ SWZ(rb)) * 8);
  }

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  constexpr int LPW = LA + LB;   // loads per wavefront and K step
#pragma unroll
  for (int st = 0; st < 3; ++st)
#pragma unroll
    for (int i = 0; i < LPW; ++i) issue_load(i, min(st, KT - 1), st);
  // K step 0 has landed once at most the two younger steps are outstanding
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(2 * LPW) : "memory");

  bf16x8_t af[2][MI], bfr[2][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) af[0][mi] = *(const bf16x8_t*)(lds + a_fr[0] + mi * 32 * BK);
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) bfr[0][ni] = *(const bf16x8_t*)(lds + b_fr[0] + ni * 32 * BK);

  constexpr int NM = MI * NI, FR = MI + NI;
  auto iteration = [&](auto STAGE, int kt) {
    constexpr int st = decltype(STAGE)::value;            // stage being multiplied = kt % 4
    const bf16_t* cur = lds + st * STG;
    const bf16_t* nxt = lds + ((st + 1) & 3) * STG;
    const int kload = min(kt + 3, KT - 1);                 // steps past the end re-read the last one into a dead stage
    static_for<2>([&](auto KK) {
      constexpr int kk = decltype(KK)::value;
      constexpr int R = kk == 0 ? FR + LPW : FR;           // memory instructions of this sub-step
      if constexpr (kk == 1)
        asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(2 * LPW) : "memory");
      static_for<NM>([&](auto J) {
        constexpr int j = decltype(J)::value;
        constexpr int mi = j / NI, ni = j % NI;
        acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk][mi], bfr[kk][ni], acc[mi][ni], 0, 0, 0);
        constexpr int lo = j * R / NM, hi = (j + 1) * R / NM;
        static_for<hi - lo>([&](auto RR) {
          constexpr int r = lo + decltype(RR)::value;
          if constexpr (r < MI) {
            const bf16_t* src = kk == 1 ? nxt + a_fr[0] : cur + a_fr[1];
            af[kk ^ 1][r] = *(const bf16x8_t*)(src + r * 32 * BK);
          } else if constexpr (r < FR) {
            const bf16_t* src = kk == 1 ? nxt + b_fr[0] : cur + b_fr[1];
            bfr[kk ^ 1][r - MI] = *(const bf16x8_t*)(src + (r - MI) * 32 * BK);
          } else {
            issue_load(r - FR, kload, (st + 3) & 3);
          }
        });
        __builtin_amdgcn_sched_barrier(0);
      });
    });
  };
  for (int kt = 0; kt < KT; kt += 4) {
    iteration(std::integral_constant<int, 0>{}, kt);
    iteration(std::integral_constant<int, 1>{}, kt + 1);
    iteration(std::integral_constant<int, 2>{}, kt + 2);
    iteration(std::integral_constant<int, 3>{}, kt + 3);
  }
  if (has_rs && tid < BM) rs_inv[tid] = rs_mine;
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");   // no load may still be landing in LDS

  constexpr bool STAGED = true;
  constexpr int STAGE_ELEMS = NSTG * STG / NW;   // per wavefront
  bf16_t* stage = lds + wave * STAGE_ELEMS;
  gemm_epilogue<MI, NI, EPI, STAGED, STAGE_ELEMS>(g, acc, stage, b, m0 + wm * TM, n0 + wn * TN, lane, has_rs ? rs_inv + wm * TM : nullptr);
}

template <int BM, int BN, int WM, int WN, int EPI>
static int launch_dl(const pt_gemm_args& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const size_t lds = (size_t)4 * (BM + BN) * 32 * sizeof(bf16_t);
  auto kern = gemm_dl_kernel<BM, BN, WM, WN, EPI>;
  PT_SET_MAX_LDS_ONCE(kern, lds);
  const int64_t total = (int64_t)tiles_m * tiles_n * g.batch;
  if (total > 0x7fffffff) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "GEMM grid too large");
  hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(WM * WN * 64), lds, s, g, tiles_m, tiles_n);
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

template <int BM, int BN, int WM, int WN, int BK, int EPI>
static int launch_cfg(const pt_gemm_args& g, hipStream_t s) {
  const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
  const size_t lds = (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
  auto kern = gemm_mfma_kernel<BM, BN, WM, WN, BK, EPI>;
  PT_SET_MAX_LDS_ONCE(kern, lds);
  const int64_t total = (int64_t)tiles_m * tiles_n * g.batch;
  if (total > 0x7fffffff) return pt_set_error(PT_ERR_INVALID_ARGUMENT, "GEMM grid too large");
  const unsigned grid = (unsigned)total;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(WM * WN * 64), lds, s, g, tiles_m, tiles_n);
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

// One (epilogue, tile configuration) pair; the pairs are instantiated explicitly, spread over several
// translation units so that they compile in parallel.
template <int EPI, int CFG>
int pt_gemm_mfma_launch_one(const pt_gemm_args& g, hipStream_t s) {
  if constexpr (CFG == 0) return launch_cfg<256, 256, 2, 2, 64, EPI>(g, s);
  else if constexpr (CFG == 1) return launch_cfg<256, 128, 2, 2, 32, EPI>(g, s);
  else if constexpr (CFG == 2) return launch_cfg<128, 128, 2, 2, 64, EPI>(g, s);
  else if constexpr (CFG == 3) return launch_cfg<64, 256, 1, 4, 64, EPI>(g, s);
  else if constexpr (CFG == 4) return launch_cfg<128, 256, 2, 2, 64, EPI>(g, s);
  else if constexpr (CFG == 5) return launch_cfg<32, 256, 1, 4, 64, EPI>(g, s);
  else if constexpr (CFG == 6) return launch_cfg<64, 256, 1, 2, 64, EPI>(g, s);
  else if constexpr (CFG == 7) return launch_cfg<32, 256, 1, 2, 64, EPI>(g, s);
  else if constexpr (CFG == 8) return launch_cfg<128, 256, 2, 2, 32, EPI>(g, s);
  else if constexpr (CFG == 9) return launch_cfg<128, 128, 2, 2, 32, EPI>(g, s);
  else if constexpr (CFG == 10) return launch_dl<256, 256, 4, 2, EPI>(g, s);
  else return launch_dl<256, 256, 2, 2, EPI>(g, s);
}

#define PT_GEMM_INSTANTIATE(EPI, CFG) template int pt_gemm_mfma_launch_one<EPI, CFG>(const pt_gemm_args& g, hipStream_t s);

#endif  // PT_GEMM_MFMA_IMPL_H_

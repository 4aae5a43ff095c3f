// Causal flash-style prefill attention on the gfx950 matrix cores (bf16 operands, fp32 softmax).
//
// One wavefront owns 32 query rows of one (track, sequence, head) and walks the keys in blocks of
// 32.  Everything is computed transposed so that no operand ever needs a transpose:
//
//   S^T [32 keys x 32 queries] = K_blk [32 x hd] . Q^T          (A = K rows, B = Q rows; both hd-contiguous)
//   O^T [hd x 32 queries]     += V^T_blk [hd x 32 keys] . P^T   (A = rows of the V^T cache, key-contiguous;
//                                                                B = P^T straight from the S^T registers)
//
// In the S^T accumulator a lane holds one query column (lane % 32) and 16 keys, which is exactly the
// B-operand layout of the second product, so the probabilities never leave the lane's registers.  The
// softmax statistics (running max and sum) are per query = per lane; the two half-waves that share a
// query combine their maxima with one cross-lane exchange per key block.  The accumulator of O^T also
// has the query in the lane, so the online-softmax rescale is a per-lane multiply.
//
// Key order inside a block: MFMA row r of S^T is loaded from key pi(r) (r with bits 2 and 3 swapped),
// which makes the 8 probabilities a half-wave feeds to one PV MFMA eight consecutive keys - one 16-byte
// read of a V^T row.
#include <type_traits>

#include "pt_device.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}

union pk8 {
  bf16x8_t v;
  uint32_t u[4];
};

template <int HD>
__global__ void __launch_bounds__(256) attn_prefill_mfma_kernel(const pt_attn_args a) {
  constexpr int KS = HD / 16;   // MFMAs per S^T block
  constexpr int HB = HD / 32;   // 32-row blocks of O^T
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int qblocks = gridDim.x;
  const int qb = qblocks - 1 - (int)blockIdx.x;   // heavy (late) query blocks first
  const int q0 = qb * 128 + wave * 32;
  if (q0 >= a.S) return;
  const int head = blockIdx.y;
  const int t = blockIdx.z / a.B, seq = blockIdx.z - t * a.B;
  const int kvh = head / (a.H / a.Hkv);
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const bf16_t* K = (const bf16_t*)a.kc + hidx * a.kv_head_elems;
  const bf16_t* Vt = (const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad);
  const int64_t row = (int64_t)seq * a.S + q0 + l32;
  const int64_t qoff = t * a.q_bstride + row * (a.H * HD) + head * HD;
  const bf16_t* qrow = (const bf16_t*)a.q + qoff;

  bf16x8_t qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = *(const bf16x8_t*)(qrow + kk * 16 + half * 8);

  const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);   // pi(l32)
  const bf16_t* kptr = K + (int64_t)krow * HD + half * 8;
  const bf16_t* vptr = Vt + (int64_t)l32 * a.s_pad + 8 * half;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);

  f32x16_t oacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[hb][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int nkb = q0 / 32 + 1;
  for (int kb = 0; kb < nkb; ++kb) {
    f32x16_t s;
#pragma unroll
    for (int v = 0; v < 16; ++v) s[v] = 0.f;
    const bf16_t* kp = kptr + (int64_t)kb * 32 * HD;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const bf16x8_t kf = *(const bf16x8_t*)(kp + kk * 16);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
    }
    // register v of this lane: key kb*32 + 16*(v/8) + 8*half + v%8, query q0 + l32
    float mx = -INFINITY;
    if (kb == nkb - 1) {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key_in = 16 * (v >> 3) + 8 * half + (v & 7);
        s[v] = key_in > l32 ? -INFINITY : s[v] * scale_log2;
        mx = fmaxf(mx, s[v]);
      }
    } else {
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        s[v] *= scale_log2;
        mx = fmaxf(mx, s[v]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
    float psum = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      s[v] = __builtin_amdgcn_exp2f(s[v] - m_new);
      psum += s[v];
    }
    l_run = l_run * corr + psum;
    m_run = m_new;
    if (__any(corr != 1.0f)) {
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[hb][v] *= corr;
    }
    pk8 pf[2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) pf[u].u[i] = pack_bf16x2(s[8 * u + 2 * i], s[8 * u + 2 * i + 1]);
    const bf16_t* vp = vptr + kb * 32;
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const bf16x8_t vf = *(const bf16x8_t*)(vp + (int64_t)hb * 32 * a.s_pad + 16 * u);
        oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u].v, oacc[hb], 0, 0, 0);
      }
  }
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l;
  bf16_t* orow = (bf16_t*)a.o + qoff;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      uint2 pk;
      pk.x = pack_bf16x2(oacc[hb][vg * 4 + 0] * inv, oacc[hb][vg * 4 + 1] * inv);
      pk.y = pack_bf16x2(oacc[hb][vg * 4 + 2] * inv, oacc[hb][vg * 4 + 3] * inv);
      *(uint2*)(orow + hb * 32 + 8 * vg + 4 * half) = pk;
    }
}


// ------------------------------------------------------------------------------------------------
// LDS-tiled variant (prefill lengths that are a multiple of 64).  A workgroup of 4 wavefronts owns 128
// query rows of one (track, sequence, head); each wavefront 32 of them.  Keys and values are walked in
// tiles of 64 positions that are staged once per workgroup in LDS (K tile [64][hd], V^T tile [hd][64],
// 16-byte chunks XOR-swizzled so that 16 lanes reading 16 different rows never share a bank) and read by
// all four wavefronts; the next tile travels from global memory through registers while the current one
// is multiplied.  Per tile a wavefront issues 2*hd/16 MFMAs for S^T and hd/32*4 for O^T; the softmax
// uses one fused multiply-add and one exp2 per score.  The MFMA operand fragments come from LDS through a ring of
// PF registers, PF reads ahead of the MFMA that needs them (measured at 16 heads x 128, 4096 tokens: 755 TFLOP/s
// with every read waited for in front of its MFMA, 822 with two in flight, 836 with four; deeper rings add nothing).
// ------------------------------------------------------------------------------------------------
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <int HD, int PF>   // PF: operand fragments in flight between LDS and the matrix cores
__global__ void __launch_bounds__(256, HD == 64 ? 3 : 2) attn_prefill_lds_kernel(const pt_attn_args a, int nqb) {
  constexpr int KS = HD / 16;          // MFMAs per 32-key block of S^T
  constexpr int HB = HD / 32;          // 32-row blocks of O^T
  constexpr int KCPR = HD / 8;         // 16-byte chunks per K row
  constexpr int KCH = 64 * KCPR / 256; // K chunks per thread and tile
  constexpr int VCH = HD * 8 / 256;    // V^T chunks per thread and tile (rows of 64 positions = 8 chunks)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16_t* Ks = (bf16_t*)smem;              // [2][64][HD]
  bf16_t* Vs = Ks + 2 * 64 * HD;           // [2][HD][64]
  auto kswz = [](int row) { return HD == 64 ? ((row >> 1) & 7) : (row & 15); };
  auto vswz = [](int row) { return (row >> 1) & 7; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  // Workgroup ids are dealt round-robin to the 8 XCDs.  A (track, sequence, head) combination keeps
  // all its query blocks on one XCD (its K/V stay in that L2) and every XCD gets the same mix of
  // long (late) and short (early) query blocks; long ones first.
  const int combos = a.n_tracks * a.B * a.H;
  int combo, qb;
  if ((combos & 7) == 0) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    combo = xcd + 8 * (j / nqb);
    qb = nqb - 1 - (j % nqb);
  } else {
    combo = blockIdx.x / nqb;
    qb = nqb - 1 - (blockIdx.x % nqb);
  }
  const int q0 = qb * 128 + wave * 32;
  const int head = combo % a.H;
  const int tb = combo / a.H;
  const int t = tb / a.B, seq = tb - t * a.B;
  const int kvh = head / (a.H / a.Hkv);
  // rows of this sequence: S of them from row seq * S, or (ragged batch) its padded length from its first packed row
  int64_t row0 = (int64_t)seq * a.S;
  int slen = a.S;
  if (a.seq_info) {
    const int4 si = a.seq_info[seq];
    row0 = si.x;
    slen = si.y;
    if (qb * 128 >= slen) return;         // a shorter sequence has fewer query blocks (whole workgroup)
  }
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const bf16_t* K = (const bf16_t*)a.kc + hidx * a.kv_head_elems;
  const bf16_t* Vt = (const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad);
  const bool active = q0 < slen;           // the last workgroup of a sequence may be partly empty
  const int64_t row = row0 + min(q0 + l32, slen - 1);
  const int64_t qoff = t * a.q_bstride + row * (a.H * HD) + head * HD;

  bf16x8_t qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = *(const bf16x8_t*)((const bf16_t*)a.q + qoff + kk * 16 + half * 8);

  // staging: K tile chunk id = tid + i*256 -> row id / KCPR, chunk id % KCPR; V^T likewise with 8 chunks per row
  const bf16_t* k_src[KCH];
  const bf16_t* v_src[VCH];
  int k_dst[KCH], v_dst[VCH];
#pragma unroll
  for (int i = 0; i < KCH; ++i) {
    const int id = tid + i * 256, r = id / KCPR, c = id % KCPR;
    k_src[i] = K + (int64_t)r * HD + c * 8;
    k_dst[i] = r * HD + ((c ^ kswz(r)) * 8);
  }
#pragma unroll
  for (int i = 0; i < VCH; ++i) {
    const int id = tid + i * 256, r = id >> 3, c = id & 7;
    v_src[i] = Vt + (int64_t)r * a.s_pad + c * 8;
    v_dst[i] = r * 64 + ((c ^ vswz(r)) * 8);
  }
  u32x4_t k_reg[KCH], v_reg[VCH];

  // fragment addresses inside a tile
  const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);   // MFMA row r of S^T holds key pi(r)
  int k_fr[2][KS];    // [32-key block][hd step]
#pragma unroll
  for (int rb = 0; rb < 2; ++rb)
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      const int r = rb * 32 + krow;
      k_fr[rb][kk] = r * HD + (((kk * 2 + half) ^ kswz(r)) * 8);
    }
  int v_fr[4];        // [16-key step]: chunk 2*step + half of row l32 (+32*hb rows: same swizzle since 32 % 16 == 0)
#pragma unroll
  for (int st = 0; st < 4; ++st) v_fr[st] = l32 * 64 + (((st * 2 + half) ^ vswz(l32)) * 8);

  const float c_log2 = 1.4426950408889634f / sqrtf((float)HD);
  f32x16_t oacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[hb][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;   // running max of the raw scores, running sum

  const int ntiles = min((qb * 128 + 128), slen) / 64;     // key tiles this workgroup walks
#pragma unroll
  for (int i = 0; i < KCH; ++i) k_reg[i] = *(const u32x4_t*)(k_src[i]);
#pragma unroll
  for (int i = 0; i < VCH; ++i) v_reg[i] = *(const u32x4_t*)(v_src[i]);
#pragma unroll
  for (int i = 0; i < KCH; ++i) *(u32x4_t*)(Ks + k_dst[i]) = k_reg[i];
#pragma unroll
  for (int i = 0; i < VCH; ++i) *(u32x4_t*)(Vs + v_dst[i]) = v_reg[i];
  __syncthreads();

  for (int kt = 0; kt < ntiles; ++kt) {
    const int cur = kt & 1;
    const bf16_t* Kc = Ks + cur * 64 * HD;
    const bf16_t* Vc = Vs + cur * HD * 64;
    const int nxt = min(kt + 1, ntiles - 1);   // the last iteration re-reads its own tile; the copy is unused
#pragma unroll
    for (int i = 0; i < KCH; ++i) k_reg[i] = *(const u32x4_t*)(k_src[i] + (int64_t)nxt * 64 * HD);
#pragma unroll
    for (int i = 0; i < VCH; ++i) v_reg[i] = *(const u32x4_t*)(v_src[i] + nxt * 64);
    __builtin_amdgcn_sched_barrier(0);

    if (active && kt * 64 <= q0 + 31) {       // wave-uniform: tiles entirely above the diagonal are skipped
      f32x16_t s[2];
      const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      // Operand fragments travel through a ring of PF registers: the LDS read of fragment i + PF is issued right
      // behind the MFMA that consumed fragment i, so a read has PF MFMAs to arrive instead of being waited for in
      // front of its own MFMA (the fences keep the compiler from moving the reads back).
      bf16x8_t fr[PF];
#pragma unroll
      for (int i = 0; i < PF; ++i) fr[i] = *(const bf16x8_t*)(Kc + k_fr[i / KS][i % KS]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 2 * KS; ++i) {
        const int rb = i / KS, kk = i % KS;
        // the first product takes the constant 0 as its addend: no register zeroing
        s[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[i % PF], qf[kk], kk == 0 ? zero16 : s[rb], 0, 0, 0);
        if (i + PF < 2 * KS) fr[i % PF] = *(const bf16x8_t*)(Kc + k_fr[(i + PF) / KS][(i + PF) % KS]);
        else fr[i % PF] = *(const bf16x8_t*)(Vc + ((i + PF - 2 * KS) / 4) * 32 * 64 + v_fr[(i + PF - 2 * KS) % 4]);   // first V^T fragments: they do not wait for the softmax
        __builtin_amdgcn_sched_barrier(0);
      }
      // register v of block rb: key kt*64 + rb*32 + 16*(v/8) + 8*half + v%8, query q0 + l32
      if (kt * 64 + 63 > q0) {                // the tile touches the diagonal: mask
        const int qrel = q0 + l32 - kt * 64;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
          for (int v = 0; v < 16; ++v)
            if (rb * 32 + 16 * (v >> 3) + 8 * half + (v & 7) > qrel) s[rb][v] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[rb][v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      // The reference of the exponentials moves to the new maximum only when that exceeds the old reference by
      // more than 8 binary orders (always on the first tile, where the reference is -inf); until then the
      // probabilities stay below 2^8 relative to the reference, which fp32 sums and bf16 operands hold without
      // loss, and the accumulators need no rescaling.  Both half-waves of a query see the same mx.
      const bool grow = (mx - m_run) * c_log2 > 8.0f;
      if (__any(grow)) {
        const float m_new = grow ? mx : m_run;
        const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
        l_run *= corr;
        m_run = m_new;
#pragma unroll
        for (int hb = 0; hb < HB; ++hb)
#pragma unroll
          for (int v = 0; v < 16; ++v) oacc[hb][v] *= corr;
      }
      const float mc = m_run * c_log2;
      float psum = 0.f;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          s[rb][v] = __builtin_amdgcn_exp2f(fmaf(s[rb][v], c_log2, -mc));
          psum += s[rb][v];
        }
      l_run += psum;
      pk8 pf[4];   // 16-key steps: (rb, u) -> rb*2 + u
#pragma unroll
      for (int st = 0; st < 4; ++st)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          pf[st].u[i] = pack_bf16x2(s[st >> 1][8 * (st & 1) + 2 * i], s[st >> 1][8 * (st & 1) + 2 * i + 1]);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < HB * 4; ++i) {
        const int hb = i / 4, st = i % 4;
        oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[(i + 2 * KS) % PF], pf[st].v, oacc[hb], 0, 0, 0);
        if (i + PF < HB * 4) fr[(i + 2 * KS) % PF] = *(const bf16x8_t*)(Vc + ((i + PF) / 4) * 32 * 64 + v_fr[(i + PF) % 4]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    bf16_t* Kn = Ks + (cur ^ 1) * 64 * HD;
    bf16_t* Vn = Vs + (cur ^ 1) * HD * 64;
#pragma unroll
    for (int i = 0; i < KCH; ++i) *(u32x4_t*)(Kn + k_dst[i]) = k_reg[i];
#pragma unroll
    for (int i = 0; i < VCH; ++i) *(u32x4_t*)(Vn + v_dst[i]) = v_reg[i];
    __syncthreads();
  }
  if (!active) return;
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l;
  bf16_t* orow = (bf16_t*)a.o + qoff;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      uint2 pk;
      pk.x = pack_bf16x2(oacc[hb][vg * 4 + 0] * inv, oacc[hb][vg * 4 + 1] * inv);
      pk.y = pack_bf16x2(oacc[hb][vg * 4 + 2] * inv, oacc[hb][vg * 4 + 3] * inv);
      *(uint2*)(orow + hb * 32 + 8 * vg + 4 * half) = pk;
    }
}

// ------------------------------------------------------------------------------------------------
// Software-pipelined form of the LDS-tiled kernel.  Same tiling (128 queries per workgroup, 32 per wavefront, key
// tiles of 64, transposed products), but the two matrix products of a tile no longer wait for the softmax between
// them; a wavefront issues instructions in order, so vector work only overlaps matrix work when the two are
// interleaved in the instruction stream:
//   phase A  the score product of tile t+1 (K_{t+1} . Q^T) is issued one MFMA at a time, and after every MFMA a
//            slice of tile t's softmax (scale, exp2, row sum, bf16 packing) follows;
//   phase B  the value product of tile t (V^T_t . P^T_t) is issued the same way, with the running-maximum search
//            over the fresh scores of tile t+1 between its MFMAs.
// K and V^T tiles arrive by direct global -> LDS loads (no staging registers, which the second set of score
// registers needs), two tiles ahead for K and one ahead for V^T, with one barrier per tile.
// ------------------------------------------------------------------------------------------------
template <int HD, int NW, int NSTG>
__global__ void __launch_bounds__(NW * 64, 2) attn_prefill_pipe_kernel(const pt_attn_args a, int nqb) {
  constexpr int QB = NW * 32;           // queries per workgroup
  constexpr int LEAD = NSTG - 1;        // tiles a load is issued ahead of its use
  constexpr int KS = HD / 16;           // MFMAs per 32-key block of S^T
  constexpr int HB = HD / 32;           // 32-row blocks of O^T
  constexpr int NS = 2 * KS;            // score MFMAs per tile
  constexpr int NPV = HB * 4;           // value MFMAs per tile
  constexpr int KROWB = HD * 2;         // bytes of a K row
  constexpr int K_CPR = KROWB / 16;     // 16-byte chunks per K row
  constexpr int K_RPI = 64 / K_CPR;     // K rows per direct-load instruction (64 lanes x 16 B = 1 KiB)
  constexpr int K_NI = 64 / K_RPI / NW; // direct-load instructions per wavefront for a K tile
  constexpr int V_NI = HD / 8 / NW;     // ... for a V^T tile (rows of 128 B: 8 per instruction)
  static_assert(K_NI >= 1 && V_NI >= 1, "more wavefronts than direct-load instructions per tile");
  constexpr int TILE_B = 64 * HD * 2;   // bytes of a K tile = bytes of a V^T tile
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  unsigned char* Ks = smem;                     // [NSTG][64][HD]
  unsigned char* Vs = smem + NSTG * TILE_B;     // [NSTG][HD][64]
  auto kswz = [](int row) { return HD == 64 ? ((row >> 1) & 7) : (row & 15); };
  auto vswz = [](int row) { return (row >> 1) & 7; };

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int combos = a.n_tracks * a.B * a.H;
  int combo, qb;
  if ((combos & 7) == 0) {
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    combo = xcd + 8 * (j / nqb);
    qb = nqb - 1 - (j % nqb);
  } else {
    combo = blockIdx.x / nqb;
    qb = nqb - 1 - (blockIdx.x % nqb);
  }
  const int q0 = qb * QB + wave * 32;
  const int head = combo % a.H;
  const int tb = combo / a.H;
  const int t_ = tb / a.B, seq = tb - t_ * a.B;
  const int kvh = head / (a.H / a.Hkv);
  int64_t row0 = (int64_t)seq * a.S;
  int slen = a.S;
  if (a.seq_info) {
    const int4 si = a.seq_info[seq];
    row0 = si.x;
    slen = si.y;
    if (qb * QB >= slen) return;
  }
  const int64_t hidx = t_ * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const char* K = (const char*)((const bf16_t*)a.kc + hidx * a.kv_head_elems);
  const char* Vt = (const char*)((const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad));
  const bool active = q0 < slen;
  const int64_t row = row0 + min(q0 + l32, slen - 1);
  const int64_t qoff = t_ * a.q_bstride + row * (a.H * HD) + head * HD;

  bf16x8_t qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) qf[kk] = *(const bf16x8_t*)((const bf16_t*)a.q + qoff + kk * 16 + half * 8);

  const int ntiles = min(qb * QB + QB, slen) / 64;                // key tiles the workgroup walks
  const int nt_w = active ? min(ntiles, (q0 + 31) / 64 + 1) : 0;  // ... of which this wavefront needs the first nt_w

  // direct loads: instruction i of this wavefront covers rows (wave * NI + i) * RPI ... of the tile; a lane fetches
  // the logical chunk that belongs at its LDS position under the XOR swizzle
  typedef const __attribute__((address_space(1))) void* gptr_t;
  typedef __attribute__((address_space(3))) void* lptr_t;
  uint32_t k_off[K_NI], v_off[V_NI];
#pragma unroll
  for (int i = 0; i < K_NI; ++i) {
    const int r = (wave * K_NI + i) * K_RPI + lane / K_CPR;
    k_off[i] = (uint32_t)(r * KROWB + (((lane % K_CPR) ^ kswz(r)) * 16));
  }
#pragma unroll
  for (int i = 0; i < V_NI; ++i) {
    const int r = (wave * V_NI + i) * 8 + (lane >> 3);
    v_off[i] = (uint32_t)(r * a.s_pad * 2 + (((lane & 7) ^ vswz(r)) * 16));
  }
  auto load_k = [&](int tile, int buf) {
#pragma unroll
    for (int i = 0; i < K_NI; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(K + (size_t)tile * TILE_B + k_off[i]),
                                       (lptr_t)(Ks + buf * TILE_B + (wave * K_NI + i) * 1024), 16, 0, 0);
  };
  auto load_v = [&](int tile, int buf) {
#pragma unroll
    for (int i = 0; i < V_NI; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(Vt + (size_t)tile * 128 + v_off[i]),
                                       (lptr_t)(Vs + buf * TILE_B + (wave * V_NI + i) * 1024), 16, 0, 0);
  };

  // fragment addresses: K row pi(l32) (+32 for the second block), 16-byte chunk (2 kk + half) ^ swizzle; the swizzle of
  // a lane's row is the same in both blocks, so one XOR with a per-lane constant forms every chunk index
  const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);   // MFMA row r of S^T holds key pi(r)
  const int k_base = krow * KROWB, k_x = half ^ kswz(krow);
  const int v_base = l32 * 128, v_x = half ^ vswz(l32);                  // rows l32 + 32 hb share the swizzle
  auto k_frag = [&](const unsigned char* Kt, int j) {   // j = rb * KS + kk
    const int rb = j / KS, kk = j % KS;
    return *(const bf16x8_t*)(Kt + rb * 32 * KROWB + k_base + (((2 * kk) ^ k_x) * 16));
  };
  auto v_frag = [&](const unsigned char* Vtile, int j) {   // j = hb * 4 + st
    const int hb = j / 4, st = j % 4;
    return *(const bf16x8_t*)(Vtile + hb * 32 * 128 + v_base + (((2 * st) ^ v_x) * 16));
  };

  const float c_log2 = 1.4426950408889634f / sqrtf((float)HD);
  const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16_t oacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb) oacc[hb] = zero16;
  float m_run = -INFINITY, l_run = 0.f;

  // register v of score block rb: key tile * 64 + rb * 32 + 16 (v / 8) + 8 half + v % 8, query q0 + l32
  auto mask_tile = [&](f32x16_t (&s)[2], int tile) {
    if (tile * 64 + 63 > q0) {
      const int qrel = q0 + l32 - tile * 64;
#pragma unroll
      for (int rb = 0; rb < 2; ++rb)
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (rb * 32 + 16 * (v >> 3) + 8 * half + (v & 7) > qrel) s[rb][v] = -INFINITY;
    }
  };
  // The reference of the exponentials moves to a new maximum only when that exceeds it by more than 8 binary orders
  // (always on the first tile); until then the probabilities stay below 2^8, which fp32 sums and bf16 operands hold,
  // and the accumulators need no rescaling.
  auto new_reference = [&](float mx) {
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const bool grow = (mx - m_run) * c_log2 > 8.0f;
    if (__any(grow)) {
      const float m_new = grow ? mx : m_run;
      const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
      l_run *= corr;
      m_run = m_new;
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[hb][v] *= corr;
    }
  };

  // prologue: V^T of tiles 0 .. LEAD-1 and K of tiles 0 .. LEAD into LDS (tile u lives in stage u % NSTG), scores of tile 0
#pragma unroll
  for (int u = 0; u < NSTG; ++u) {
    if (u < ntiles) load_k(u, u);
    if (u < LEAD && u < ntiles) load_v(u, u);
  }
  asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  f32x16_t s_a[2], s_b[2];
  if (nt_w > 0) {
#pragma unroll
    for (int j = 0; j < NS; ++j) s_a[j / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k_frag(Ks, j), qf[j % KS], j % KS == 0 ? zero16 : s_a[j / KS], 0, 0, 0);
    mask_tile(s_a, 0);
    float mx = -INFINITY;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb)
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s_a[rb][v]);
    new_reference(mx);
  }
  __syncthreads();   // every wavefront has read tile 0 of K: its buffer may be refilled

  // one tile: s_cur holds the scores of tile t (reference already moved), s_nxt receives those of tile t + 1.
  // NXT: this wavefront also needs tile t + 1.  Operand fragments are read from LDS three MFMAs ahead.
  constexpr int PF = 3;   // fragment ring depth
  auto compute = [&](auto NXT_, f32x16_t (&s_cur)[2], f32x16_t (&s_nxt)[2], const unsigned char* Kn, const unsigned char* Vc, int t) {
    constexpr bool NXT = decltype(NXT_)::value;
    const float mc = m_run * c_log2;
    float psum = 0.f;
    pk8 pf[4];
    bf16x8_t fr[PF];
    // ---- phase A: score MFMAs of tile t + 1, a slice of tile t's exponentials after each
    constexpr int CH = 32 / NS;   // scores per slice
    if constexpr (NXT) {
#pragma unroll
      for (int j = 0; j < PF - 1; ++j) fr[j] = k_frag(Kn, j);
    }
    static_for<NS>([&](auto J) {
      constexpr int j = decltype(J)::value;
      if constexpr (NXT) {
        if constexpr (j + PF - 1 < NS) fr[(j + PF - 1) % PF] = k_frag(Kn, j + PF - 1);
        s_nxt[j / KS] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % PF], qf[j % KS], j % KS == 0 ? zero16 : s_nxt[j / KS], 0, 0, 0);
      }
      static_for<CH / 2>([&](auto C_) {
        constexpr int idx = j * CH + 2 * decltype(C_)::value;   // score pair (idx, idx + 1): block idx / 16, register idx % 16
        constexpr int rb = idx / 16, v = idx % 16;
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s_cur[rb][v], c_log2, -mc));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s_cur[rb][v + 1], c_log2, -mc));
        psum += p0 + p1;
        pf[idx / 8].u[(idx % 8) / 2] = pack_bf16x2(p0, p1);
      });
      __builtin_amdgcn_sched_barrier(0);
    });
    l_run += psum;
    // ---- phase B: value MFMAs of tile t, a slice of the maximum search over tile t + 1 after each
    if constexpr (NXT) mask_tile(s_nxt, t + 1);
    float mx = -INFINITY;
    constexpr int MCH = 32 / NPV;
#pragma unroll
    for (int j = 0; j < PF - 1; ++j) fr[j] = v_frag(Vc, j);
    static_for<NPV>([&](auto J) {
      constexpr int j = decltype(J)::value;
      if constexpr (j + PF - 1 < NPV) fr[(j + PF - 1) % PF] = v_frag(Vc, j + PF - 1);
      oacc[j / 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fr[j % PF], pf[j % 4].v, oacc[j / 4], 0, 0, 0);
      if constexpr (NXT) {
        static_for<MCH>([&](auto C_) {
          constexpr int idx = j * MCH + decltype(C_)::value;
          mx = fmaxf(mx, s_nxt[idx / 16][idx % 16]);
        });
      }
      __builtin_amdgcn_sched_barrier(0);
    });
    if constexpr (NXT) new_reference(mx);
  };
  auto iteration = [&](f32x16_t (&s_cur)[2], f32x16_t (&s_nxt)[2], int t) {
    // K of tile t + LEAD + 1 replaces K of tile t (read one iteration ago), V^T of tile t + LEAD that of tile t - 1
    const bool more_k = t + LEAD + 1 < ntiles, more_v = t + LEAD < ntiles;
    if (more_k) load_k(t + LEAD + 1, (t + LEAD + 1) % NSTG);
    if (more_v) load_v(t + LEAD, (t + LEAD) % NSTG);
    const unsigned char* Kn = Ks + ((t + 1) % NSTG) * TILE_B;
    const unsigned char* Vc = Vs + (t % NSTG) * TILE_B;
    if (t + 1 < nt_w) compute(std::true_type{}, s_cur, s_nxt, Kn, Vc, t);
    else if (t < nt_w) compute(std::false_type{}, s_cur, s_nxt, Kn, Vc, t);
    // the next iteration needs K of tile t + 2 and V^T of tile t + 1: everything but the loads of the last LEAD - 1
    // iterations (loads complete in order); near the end, where fewer loads are issued, simply everything
    if (more_k && more_v) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"((LEAD - 1) * (K_NI + V_NI)) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
  };
  for (int t = 0; t < ntiles; t += 2) {
    iteration(s_a, s_b, t);
    if (t + 1 < ntiles) iteration(s_b, s_a, t + 1);
  }
  if (!active) return;
  const float l = l_run + __shfl_xor(l_run, 32, 64);
  const float inv = 1.0f / l;
  bf16_t* orow = (bf16_t*)a.o + qoff;
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      uint2 pk;
      pk.x = pack_bf16x2(oacc[hb][vg * 4 + 0] * inv, oacc[hb][vg * 4 + 1] * inv);
      pk.y = pack_bf16x2(oacc[hb][vg * 4 + 2] * inv, oacc[hb][vg * 4 + 3] * inv);
      *(uint2*)(orow + hb * 32 + 8 * vg + 4 * half) = pk;
    }
}

// 0: the plain LDS-tiled kernel (default), 1: the software-pipelined kernel (pt_set_tuning).  Measured on the
// Large PT shape (16 heads x 128, 8 x 4096 tokens, 8 tracks): 5.5 ms per launch for the plain kernel, 7.3 - 7.9 ms for
// the pipelined one, so the plain kernel stays the default.
int pt_tune_attn_prefill = 0;

template <int HD>
static int launch_lds(const pt_attn_args& a, hipStream_t s) {
  const int slen_max = a.seq_info ? a.max_plen : a.S;
  if (pt_tune_attn_prefill == 1) {
    // software-pipelined kernel: 8 wavefronts (256 queries) per workgroup, four K / V^T stages in LDS
    constexpr int NW = 8, NSTG = 4;
    const int nqb = (slen_max + NW * 32 - 1) / (NW * 32);
    const int64_t total = (int64_t)a.n_tracks * a.B * a.H * nqb;
    if (total > 0x7fffffff) return 0;
    const size_t lds = (size_t)NSTG * 2 * 64 * HD * sizeof(bf16_t);
    auto kern = attn_prefill_pipe_kernel<HD, NW, NSTG>;
    PT_SET_MAX_LDS_ONCE(kern, lds);
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(NW * 64), lds, s, a, nqb);
    PT_HIP_CHECK(hipGetLastError());
    return 1;
  }
  const int nqb = (slen_max + 127) / 128;
  const int64_t total = (int64_t)a.n_tracks * a.B * a.H * nqb;
  if (total > 0x7fffffff) return 0;
  const dim3 grid((unsigned)total);
  const size_t lds = (size_t)2 * (64 * HD + HD * 64) * sizeof(bf16_t);
  {
    auto kern = attn_prefill_lds_kernel<HD, 4>;
    PT_SET_MAX_LDS_ONCE(kern, lds);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, s, a, nqb);
  }
  PT_HIP_CHECK(hipGetLastError());
  return 1;
}

int pt_launch_attn_prefill_mfma(const pt_attn_args& a, hipStream_t s) {
  if (a.dtype != PT_BF16 || a.pos0 != 0) return 0;
  if (a.hd != 64 && a.hd != 128) return 0;
  if (a.seq_info) {   // ragged batch: every padded length is a multiple of 64, which the LDS-tiled kernel walks
    if ((a.s_pad & 7) || (a.q_bstride & 7) || (((uintptr_t)a.q | (uintptr_t)a.o | (uintptr_t)a.kc | (uintptr_t)a.vc) & 15)) return 0;
    return a.hd == 64 ? launch_lds<64>(a, s) : launch_lds<128>(a, s);
  }
  if (a.S < 32 || a.S % 32) return 0;
  if ((a.q_bstride & 7) || (((uintptr_t)a.q | (uintptr_t)a.o | (uintptr_t)a.kc | (uintptr_t)a.vc) & 15)) return 0;
  const int64_t z = (int64_t)a.n_tracks * a.B;
  if (z > 65535 || a.H > 65535) return 0;
  dim3 grid((unsigned)((a.S + 127) / 128), (unsigned)a.H, (unsigned)z);
  if (a.S % 64 == 0 && (a.s_pad & 7) == 0) return a.hd == 64 ? launch_lds<64>(a, s) : launch_lds<128>(a, s);
  if (a.hd == 64)
    hipLaunchKernelGGL(attn_prefill_mfma_kernel<64>, grid, dim3(256), 0, s, a);
  else
    hipLaunchKernelGGL(attn_prefill_mfma_kernel<128>, grid, dim3(256), 0, s, a);
  PT_HIP_CHECK(hipGetLastError());
  return 2;
}

// Split-K decode attention over the contiguous KV cache (bf16 cache, fp32 arithmetic).
//
// One query row per (track, sequence, head).  The work is HBM-bound.  Two kernels: a matrix-core kernel
// (further down; groups of up to 32 query heads per KV head) and this vector kernel for larger groups,
// which reads the cache once per query head with 16-byte loads.  A workgroup owns one key range ("split")
// of one head:
//   phase 1  scores: a key row (hd contiguous) is covered by hd/8 lanes, 8 elements each; the partial
//            dot products are folded with cross-lane exchanges and the score goes to LDS;
//   phase 2  exact softmax numerators over the range (max, then exp2, then sum) in LDS;
//   phase 3  values: the cache holds V transposed (positions contiguous), so a lane reads 8
//            consecutive positions of one hd-row per load and multiplies them with 8 probabilities
//            from LDS; each wavefront owns hd/4 rows and reduces across lanes once at the end.
// With more than one split each workgroup writes (max, sum, unnormalised output) and a small kernel
// combines the splits; with one split the normalised output is written directly.
#include "pt_device.h"

#define DEC_CHUNK 512          // positions one wavefront covers per step of phase 3 (64 lanes x 8)
#define DEC_MAX_KEYS 8192      // positions per split (32 KB of scores in LDS)

template <int HD>
__global__ void __launch_bounds__(256) attn_decode_kernel(const pt_attn_args a, int nsplit, int keys_per_split) {
  constexpr int LPK = HD / 8;       // lanes per key row
  constexpr int KPI = 64 / LPK;     // key rows per wavefront load
  constexpr int RPW = HD / 4;       // V^T rows per wavefront
  extern __shared__ __attribute__((aligned(16))) float sc[];
  __shared__ float red[8];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int split = blockIdx.x, head = blockIdx.y;
  const int t = blockIdx.z / a.B, seq = blockIdx.z - t * a.B;
  const int nkeys = (a.row_map ? a.row_map[seq].y : a.pos0) + 1;   // ragged batch: this sequence's own length
  const int k0 = split * keys_per_split;
  const int k1 = min(nkeys, k0 + keys_per_split);
  const int n = k1 - k0;
  const int kvh = head / (a.H / a.Hkv);
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const bf16_t* K = (const bf16_t*)a.kc + hidx * a.kv_head_elems;
  const bf16_t* Vt = (const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad);
  const int64_t qoff = t * a.q_bstride + (int64_t)seq * (a.H * HD) + head * HD;
  float* part = a.partials + (((int64_t)blockIdx.z * a.H + head) * nsplit + split) * (HD + 2);

  if (n <= 0) {   // empty trailing split: neutral element of the combine
    if (tid == 0) { part[0] = -INFINITY; part[1] = 0.f; }
    for (int e = tid; e < HD; e += 256) part[2 + e] = 0.f;
    return;
  }

  // ---- phase 1: scores (already in log2 units)
  const int sub = lane % LPK, kslot = lane / LPK;
  float qf[8];
  {
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    const uint4 qv = *(const uint4*)((const bf16_t*)a.q + qoff + sub * 8);
    const uint32_t w[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      qf[2 * i] = __uint_as_float(w[i] << 16) * scale_log2;
      qf[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u) * scale_log2;
    }
  }
  float mx = -INFINITY;
  // key rows of this lane group, relative to k0: kfirst, kfirst + kstep, ... (4 in flight per step)
  const int kfirst = wave * KPI + kslot, kstep = 4 * KPI;
  const bf16_t* kp = K + (int64_t)k0 * HD + sub * 8;
  for (int kb = kfirst; kb < n; kb += 4 * kstep) {
    uint4 kv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (kb + u * kstep < n) kv[u] = *(const uint4*)(kp + (int64_t)(kb + u * kstep) * HD);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const bool valid = kb + u * kstep < n;
      float dot = 0.f;
      if (valid) {
        const uint32_t w[4] = {kv[u].x, kv[u].y, kv[u].z, kv[u].w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          dot = fmaf(qf[2 * i], __uint_as_float(w[i] << 16), dot);
          dot = fmaf(qf[2 * i + 1], __uint_as_float(w[i] & 0xffff0000u), dot);
        }
      }
      // the LPK lanes of a key row share kb, so they are active together
#pragma unroll
      for (int o = 1; o < LPK; o <<= 1) dot += __shfl_xor(dot, o, 64);
      if (valid) {
        if (sub == 0) sc[kb + u * kstep] = dot;
        mx = fmaxf(mx, dot);
      }
    }
  }
  mx = wave_max(mx);
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  const float M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));

  // ---- phase 2: numerators and their sum; zero the tail up to the next chunk border
  const int npad = (n + DEC_CHUNK - 1) / DEC_CHUNK * DEC_CHUNK;
  float ps = 0.f;
  for (int i = tid; i < npad; i += 256) {
    float p = 0.f;
    if (i < n) {
      p = __builtin_amdgcn_exp2f(sc[i] - M);
      ps += p;
    }
    sc[i] = p;
  }
  ps = wave_sum(ps);
  if (lane == 0) red[4 + wave] = ps;
  __syncthreads();
  const float Lsum = red[4] + red[5] + red[6] + red[7];

  // ---- phase 3: values
  float acc[RPW];
#pragma unroll
  for (int r = 0; r < RPW; ++r) acc[r] = 0.f;
  const bf16_t* vbase = Vt + (int64_t)(wave * RPW) * a.s_pad + k0;
  for (int c = lane * 8; c < n; c += DEC_CHUNK) {
    const float4 p0 = *(const float4*)(sc + c), p1 = *(const float4*)(sc + c + 4);
    const float p[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
    const bool tail = c + 8 > n;   // some of the 8 positions lie beyond the range: their cache bytes are not data
#pragma unroll
    for (int r0 = 0; r0 < RPW; r0 += 16) {
      uint4 vv[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) vv[r] = *(const uint4*)(vbase + (int64_t)(r0 + r) * a.s_pad + c);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t w[4] = {vv[r].x, vv[r].y, vv[r].z, vv[r].w};
        float s = acc[r0 + r];
        if (!tail) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            s = fmaf(p[2 * i], __uint_as_float(w[i] << 16), s);
            s = fmaf(p[2 * i + 1], __uint_as_float(w[i] & 0xffff0000u), s);
          }
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            if (c + 2 * i < n) s = fmaf(p[2 * i], __uint_as_float(w[i] << 16), s);
            if (c + 2 * i + 1 < n) s = fmaf(p[2 * i + 1], __uint_as_float(w[i] & 0xffff0000u), s);
          }
        }
        acc[r0 + r] = s;
      }
    }
  }
#pragma unroll
  for (int r = 0; r < RPW; ++r) acc[r] = wave_sum(acc[r]);

  if (nsplit == 1) {
    const float inv = 1.0f / Lsum;
    bf16_t* o = (bf16_t*)a.o + qoff + wave * RPW;
#pragma unroll
    for (int r = 0; r < RPW; ++r)
      if (lane == (r & 63)) o[r] = f32_to_bf16(acc[r] * inv);
  } else {
    if (tid == 0) { part[0] = M; part[1] = Lsum; }
#pragma unroll
    for (int r = 0; r < RPW; ++r)
      if (lane == (r & 63)) part[2 + wave * RPW + r] = acc[r];
  }
}

// Combines the splits of one (track, sequence, head): o = sum_s o_s 2^(m_s - M) / sum_s l_s 2^(m_s - M).
__global__ void __launch_bounds__(64) attn_decode_combine_kernel(const pt_attn_args a, int nsplit) {
  const int head = blockIdx.x;
  const int t = blockIdx.y / a.B, seq = blockIdx.y - t * a.B;
  const int hd = a.hd;
  const float* part = a.partials + ((int64_t)blockIdx.y * a.H + head) * nsplit * (hd + 2);
  float M = -INFINITY;
  for (int s = 0; s < nsplit; ++s) M = fmaxf(M, part[s * (hd + 2)]);
  float L = 0.f;
  for (int s = 0; s < nsplit; ++s) L += part[s * (hd + 2) + 1] * __builtin_amdgcn_exp2f(part[s * (hd + 2)] - M);
  const float inv = 1.0f / L;
  bf16_t* o = (bf16_t*)a.o + t * a.q_bstride + (int64_t)seq * (a.H * hd) + head * hd;
  for (int e = threadIdx.x; e < hd; e += 64) {
    float acc = 0.f;
    for (int s = 0; s < nsplit; ++s)
      acc += part[s * (hd + 2) + 2 + e] * __builtin_amdgcn_exp2f(part[s * (hd + 2)] - M);
    o[e] = f32_to_bf16(acc * inv);
  }
}

// ------------------------------------------------------------------------------------------------
// Matrix-core kernel, used whenever G = H / Hkv <= 32 (the kernel above serves larger groups): the G
// query heads that share a KV head (G = 1: plain multi-head attention) are processed together, so every
// key and value element is read exactly once.
//
//   S^T [32 keys x G] = K_blk [32 x hd] . Q^T       (A = key rows straight from the cache, B = the G queries)
//   O^T [hd x G]     += V^T_blk [hd x 32] . P^T     (A = rows of the V^T cache, B = P^T from the S^T registers)
//
// which is the prefill formulation with the query heads of a group in place of query positions (MFMA
// column = query head, padded to 32).  A workgroup owns one key range of one (track, sequence, KV head);
// its 4 wavefronts take the 32-key blocks of the range round-robin, each with its own online-softmax
// state, and merge the four states through LDS.  The cache is read by the whole workgroup in tiles of 128
// keys as 16-byte pieces of whole cache lines and handed to the MFMAs through LDS: lane-per-row loads in
// operand layout touch 32 cache lines per instruction and hold the CU's memory path below what HBM delivers.
// ------------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

union dpk8 {
  bf16x8_t v;
  uint32_t u[4];
};

#define DEC_GMAX 32

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Tiles of 128 keys: K [128 x hd] (one contiguous piece of the cache) and V^T [hd x 128] are read by the whole
// workgroup as 16-byte pieces of whole cache lines, held in registers while the previous tile is multiplied,
// and parked in LDS (two buffers for hd = 128; one for hd = 64, where a third resident workgroup covers the
// extra barrier; 16-byte chunk c of row r sits at position c ^ swizzle(r)); wavefront w then
// works on keys 32w .. 32w+31 of the tile with fragments read from LDS.
template <int HD>
__global__ void __launch_bounds__(256) attn_decode_tiled_kernel(const pt_attn_args a, int nsplit, int keys_per_split) {
  constexpr int KS = HD / 16, HB = HD / 32;
  constexpr int KROW = HD * 2;                  // bytes of a key row
  constexpr int KCH = KROW / 16;                // 16-byte chunks per key row
  constexpr int TILE = 128 * KROW;              // bytes of the K tile = bytes of the V^T tile (hd rows x 256 B)
  constexpr int NLD = TILE / 16 / 256;          // 16-byte pieces per thread and operand
  constexpr int NBUF = HD == 64 ? 1 : 2;        // LDS buffers: one (and three workgroups per CU) or two
  extern __shared__ __attribute__((aligned(1024))) char smem[];   // 2 buffers x (K tile + V^T tile)
  float (*red_o)[HD][DEC_GMAX] = (float (*)[HD][DEC_GMAX])smem;   // reuses the tiles after the key loop
  __shared__ float red_m[4][32], red_l[4][32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l32 = lane & 31, half = lane >> 5;
  const int split = blockIdx.x, kvh = blockIdx.y;
  const int t = blockIdx.z / a.B, seq = blockIdx.z - t * a.B;
  const int G = a.H / a.Hkv;
  const int nkeys = (a.row_map ? a.row_map[seq].y : a.pos0) + 1;   // ragged batch: this sequence's own length
  const int k0 = split * keys_per_split;
  const int k1 = min(nkeys, k0 + keys_per_split);
  if (k0 >= nkeys) {
    // a shorter sequence of a ragged batch has no key in this range: the neutral element of the combine
    // (whole workgroup, ahead of every barrier; split 0 is never empty)
    for (int e = tid; e < HD * G; e += 256) {
      const int g = e / HD, r = e - g * HD;
      float* part = a.partials + (((int64_t)blockIdx.z * a.H + kvh * G + g) * nsplit + split) * (HD + 2);
      if (r == 0) { part[0] = -INFINITY; part[1] = 0.f; }
      part[2 + r] = 0.f;
    }
    return;
  }
  const int64_t hidx = t * a.kv_bstride + seq * a.kv_seq_stride + kvh;
  const char* K = (const char*)((const bf16_t*)a.kc + hidx * a.kv_head_elems);
  const char* Vt = (const char*)((const bf16_t*)a.vc + hidx * ((int64_t)HD * a.s_pad));
  const int64_t qbase = t * a.q_bstride + (int64_t)seq * (a.H * HD) + (int64_t)kvh * G * HD;
  auto kswz = [](int row) { return HD == 128 ? (row & 15) : ((row >> 1) & 7); };   // K rows of 256 or 128 bytes
  auto vswz = [](int row) { return row & 15; };                                   // V^T rows of 256 bytes

  // B operand of S^T: query head l32 of the group (zero beyond G)
  bf16x8_t qf[KS];
#pragma unroll
  for (int kk = 0; kk < KS; ++kk) {
    dpk8 z;
    z.u[0] = z.u[1] = z.u[2] = z.u[3] = 0u;
    if (l32 < G) z.v = *(const bf16x8_t*)((const bf16_t*)a.q + qbase + (int64_t)l32 * HD + kk * 16 + half * 8);
    qf[kk] = z.v;
  }
  const int krow = (l32 & ~12) | ((l32 & 4) << 1) | ((l32 & 8) >> 1);   // MFMA row r of S^T holds key pi(r)
  const float c_log2 = 1.4426950408889634f / sqrtf((float)HD);

  // staging: piece i of this thread is chunk id c = tid + 256 i of the tile
  u32x4_t kreg[NLD], vreg[NLD];
  auto load_tile = [&](int kb) {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = tid + 256 * i;
      const int kr = c / KCH, kc = c - kr * KCH;                 // key row, chunk of K
      kreg[i] = *(const u32x4_t*)(K + (int64_t)min(kb + kr, k1 - 1) * KROW + kc * 16);
      const int vr = c >> 4, vc = c & 15;                        // hd row, chunk (8 keys) of V^T
      const int key = min(kb + vc * 8, (k1 - 1) & ~7);           // never past the chunk that holds the last key
      vreg[i] = *(const u32x4_t*)(Vt + ((int64_t)vr * a.s_pad + key) * 2);
    }
  };
  auto park_tile = [&](int buf, int kb) {
    char* kt = smem + buf * (2 * TILE);
    char* vt = kt + TILE;
    const bool tail = kb + 128 > k1;   // workgroup-uniform
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int c = tid + 256 * i;
      const int kr = c / KCH, kc = c - kr * KCH;
      *(u32x4_t*)(kt + kr * KROW + ((kc ^ kswz(kr)) * 16)) = kreg[i];
      const int vr = c >> 4, vc = c & 15;
      u32x4_t v = vreg[i];
      if (tail) {
        // cache bytes beyond the range are not data: zero them so that 0 * x stays 0
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int key = kb + vc * 8 + 2 * j;
          uint32_t w = v[j];
          if (key >= k1) w &= 0xffff0000u;
          if (key + 1 >= k1) w &= 0x0000ffffu;
          v[j] = w;
        }
      }
      *(u32x4_t*)(vt + vr * 256 + ((vc ^ vswz(vr)) * 16)) = v;
    }
  };

  f32x16_t oacc[HB];
#pragma unroll
  for (int hb = 0; hb < HB; ++hb)
#pragma unroll
    for (int v = 0; v < 16; ++v) oacc[hb][v] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  const int kfr_row = wave * 32 + krow;         // row of the K tile this lane multiplies
  load_tile(k0);
  park_tile(0, k0);
  __syncthreads();
  int buf = 0;
  for (int kb = k0; kb < k1; kb += 128, buf ^= (NBUF - 1)) {
    const bool more = kb + 128 < k1;
    if (more) load_tile(kb + 128);
    const char* kt = smem + buf * (2 * TILE);
    const char* vt = kt + TILE;
    const int kw = kb + wave * 32;              // first key of this wavefront's block
    if (kw < k1) {                              // wave-uniform
      f32x16_t s;
#pragma unroll
      for (int v = 0; v < 16; ++v) s[v] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KS; ++kk) {
        const bf16x8_t kf = *(const bf16x8_t*)(kt + kfr_row * KROW + (((2 * kk + half) ^ kswz(kfr_row)) * 16));
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], s, 0, 0, 0);
      }
      // register v: key kw + 16*(v/8) + 8*half + v%8, query head l32
      if (kw + 32 > k1) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          if (kw + 16 * (v >> 3) + 8 * half + (v & 7) >= k1) s[v] = -INFINITY;
      }
      float mx = -INFINITY;
#pragma unroll
      for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[v]);
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
      const float m_new = fmaxf(m_run, mx);
      const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * c_log2);
      const float mc = m_new * c_log2;
      float psum = 0.f;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        s[v] = __builtin_amdgcn_exp2f(fmaf(s[v], c_log2, -mc));
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
      dpk8 pf[2];
#pragma unroll
      for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) pf[u].u[i] = pack_bf16x2(s[8 * u + 2 * i], s[8 * u + 2 * i + 1]);
#pragma unroll
      for (int hb = 0; hb < HB; ++hb)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          const int vr = hb * 32 + l32;
          const bf16x8_t vf = *(const bf16x8_t*)(vt + vr * 256 + (((wave * 4 + 2 * u + half) ^ vswz(vr)) * 16));
          oacc[hb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[u].v, oacc[hb], 0, 0, 0);
        }
    }
    if (NBUF == 1) __syncthreads();             // one buffer: everybody is done with the tile before it is replaced
    if (more) park_tile(buf ^ (NBUF - 1), kb + 128);   // two buffers: last read while tile kb - 128 was multiplied
    __syncthreads();
  }
  // the two half-waves of a query head hold disjoint key subsets with a common running max
  l_run += __shfl_xor(l_run, 32, 64);
  // merge the four wavefront states: row (hd index) of register v in block hb = hb*32 + 8*(v/4) + 4*half + v%4
  if (half == 0) { red_m[wave][l32] = m_run; red_l[wave][l32] = l_run; }
  __syncthreads();
  float M = fmaxf(fmaxf(red_m[0][l32], red_m[1][l32]), fmaxf(red_m[2][l32], red_m[3][l32]));
  const float sc = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m_run - M) * c_log2);   // a wavefront may have had no block
  if (l32 < G) {
#pragma unroll
    for (int hb = 0; hb < HB; ++hb)
#pragma unroll
      for (int v = 0; v < 16; ++v) red_o[wave][hb * 32 + 8 * (v >> 2) + 4 * half + (v & 3)][l32] = oacc[hb][v] * sc;
  }
  __syncthreads();
  for (int e = tid; e < HD * G; e += 256) {
    const int g = e / HD, r = e - g * HD;
    float Mg = fmaxf(fmaxf(red_m[0][g], red_m[1][g]), fmaxf(red_m[2][g], red_m[3][g]));
    float L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) L += red_m[w][g] == -INFINITY ? 0.f : red_l[w][g] * __builtin_amdgcn_exp2f((red_m[w][g] - Mg) * c_log2);
    const float o = red_o[0][r][g] + red_o[1][r][g] + red_o[2][r][g] + red_o[3][r][g];
    const int head = kvh * G + g;
    if (nsplit == 1) {
      ((bf16_t*)a.o)[qbase + (int64_t)g * HD + r] = f32_to_bf16(o / L);
    } else {
      float* part = a.partials + (((int64_t)blockIdx.z * a.H + head) * nsplit + split) * (HD + 2);
      if (r == 0) { part[0] = Mg * c_log2; part[1] = L; }
      part[2 + r] = o;
    }
  }
}

template <int HD>
static int launch_gqa(const pt_attn_args& a, dim3 grid, int nsplit, int kps, hipStream_t s) {
  constexpr int LDS = (HD == 64 ? 1 : 2) * 2 * 128 * HD * 2;
  static_assert(LDS >= 4 * HD * DEC_GMAX * 4, "merge buffer must fit the tiles");
  auto kern = attn_decode_tiled_kernel<HD>;
  PT_SET_MAX_LDS_ONCE(kern, LDS);
  hipLaunchKernelGGL(kern, grid, dim3(256), LDS, s, a, nsplit, kps);
  return PT_OK;
}

int pt_launch_attn_decode(const pt_attn_args& a, hipStream_t s) {
  if (a.dtype != PT_BF16 || a.S != 1) return 0;
  if (a.hd != 64 && a.hd != 128) return 0;
  if ((a.q_bstride & 7) || (((uintptr_t)a.q | (uintptr_t)a.kc | (uintptr_t)a.vc) & 15)) return 0;
  const int64_t z = (int64_t)a.n_tracks * a.B;
  if (z > 65535 || a.H > 65535) return 0;
  const int nkeys = (a.row_map ? a.max_pos : a.pos0) + 1;   // the longest sequence decides the ranges
  const int G = a.H / a.Hkv;
  if (G <= DEC_GMAX && (a.s_pad & 7) == 0) {   // measured at least as fast as the VALU kernel for G = 1 too
    const int64_t gbase = z * a.Hkv;
    int nsplit = (int)((1024 + gbase - 1) / gbase);
    const int by_len = (nkeys + 511) / 512;
    if (nsplit > by_len) nsplit = by_len;
    if (nsplit < 1) nsplit = 1;
    if (nsplit > a.max_splits) nsplit = a.max_splits;
    int kps = (nkeys + nsplit - 1) / nsplit;
    kps = (kps + 127) / 128 * 128;
    nsplit = (nkeys + kps - 1) / kps;      // no empty split
    dim3 grid((unsigned)nsplit, (unsigned)a.Hkv, (unsigned)z);
    const int rc = a.hd == 64 ? launch_gqa<64>(a, grid, nsplit, kps, s) : launch_gqa<128>(a, grid, nsplit, kps, s);
    if (rc) return rc;
    if (nsplit > 1)
      hipLaunchKernelGGL(attn_decode_combine_kernel, dim3((unsigned)a.H, (unsigned)z), dim3(64), 0, s, a, nsplit);
    PT_HIP_CHECK(hipGetLastError());
    return 1;
  }
  const int64_t base = z * a.H;
  int nsplit = (int)((1024 + base - 1) / base);
  const int by_len = (nkeys + DEC_CHUNK - 1) / DEC_CHUNK;
  if (nsplit > by_len) nsplit = by_len;
  const int need = (nkeys + DEC_MAX_KEYS - 1) / DEC_MAX_KEYS;
  if (nsplit < need) nsplit = need;
  if (nsplit < 1) nsplit = 1;
  if (nsplit > a.max_splits) return 0;
  int kps = (nkeys + nsplit - 1) / nsplit;
  kps = (kps + DEC_CHUNK - 1) / DEC_CHUNK * DEC_CHUNK;
  if (kps > DEC_MAX_KEYS) return 0;
  const size_t lds = (size_t)kps * sizeof(float);
  dim3 grid((unsigned)nsplit, (unsigned)a.H, (unsigned)z);
  if (a.hd == 64)
    hipLaunchKernelGGL(attn_decode_kernel<64>, grid, dim3(256), lds, s, a, nsplit, kps);
  else
    hipLaunchKernelGGL(attn_decode_kernel<128>, grid, dim3(256), lds, s, a, nsplit, kps);
  if (nsplit > 1)
    hipLaunchKernelGGL(attn_decode_combine_kernel, dim3((unsigned)a.H, (unsigned)z), dim3(64), 0, s, a, nsplit);
  PT_HIP_CHECK(hipGetLastError());
  return 2;
}

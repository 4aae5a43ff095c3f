// Chooses the tile configuration of the MFMA GEMM family by shape and dispatches to the kernels, which are
// instantiated per epilogue in kernels_gemm_mfma_{store,residual,swiglu,qkv_a..d}.hip from gemm_mfma_impl.h.
#include "pt_device.h"

template <int EPI, int CFG>
int pt_gemm_mfma_launch_one(const pt_gemm_args& g, hipStream_t s);

template <int EPI>
static int launch_epi(const pt_gemm_args& g, hipStream_t s, int cfg) {
  switch (cfg) {
    case 0: return pt_gemm_mfma_launch_one<EPI, 0>(g, s);
    case 1: return pt_gemm_mfma_launch_one<EPI, 1>(g, s);
    case 2: return pt_gemm_mfma_launch_one<EPI, 2>(g, s);
    case 3: return pt_gemm_mfma_launch_one<EPI, 3>(g, s);
    case 4: return pt_gemm_mfma_launch_one<EPI, 4>(g, s);
    case 5: return pt_gemm_mfma_launch_one<EPI, 5>(g, s);
    case 6: return pt_gemm_mfma_launch_one<EPI, 6>(g, s);
    case 7: return pt_gemm_mfma_launch_one<EPI, 7>(g, s);
    case 8: return pt_gemm_mfma_launch_one<EPI, 8>(g, s);
    case 9: return pt_gemm_mfma_launch_one<EPI, 9>(g, s);
    case 10: return pt_gemm_mfma_launch_one<EPI, 10>(g, s);
    default: return pt_gemm_mfma_launch_one<EPI, 11>(g, s);
  }
}

#define GM_BK 64

// Tile configuration override for tuning runs (pt_set_tuning): -1 = choose by shape.
int pt_tune_gemm_cfg = -1;

#define GM_NCFG 12
static const int kWaveN[GM_NCFG] = {128, 64, 64, 64, 128, 64, 128, 128, 128, 64, 128, 128};   // columns per wavefront

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

// The tile configuration for a problem, or -1 if the family does not cover it (-2: nothing to do).
static int choose_cfg(const pt_gemm_args& g) {
  if (g.dtype != PT_BF16) return -1;
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return -2;
  if (g.K < 2 * GM_BK || g.K % (2 * GM_BK)) return -1;
  if ((g.lda & 7) || (g.ldb & 7) || (g.a_bstride & 7) || (g.w_bstride & 7)) return -1;
  if (((uintptr_t)g.A | (uintptr_t)g.W) & 15) return -1;
  if (g.blk_group && ((g.w_gstride & 7) || (g.M & 255))) return -1;   // expert segments are whole 256-row tiles
  if (g.a_rows && (g.a_bstride ? g.a_bstride : (int64_t)g.M * g.lda) * 2 >= ((int64_t)1 << 32)) return -1;   // 32-bit gather offsets
  if ((g.epi == EPI_STORE_F32 || g.epi == EPI_RESIDUAL) &&
      ((g.ldo & 3) || (g.N & 3) || (g.out_bstride & 3) || (g.res_bstride & 3) || (((uintptr_t)g.out | (uintptr_t)g.res) & 15))) return -1;
  if (g.epi == EPI_SWIGLU && ((g.olp_bstride & 7) || ((uintptr_t)g.olp & 15))) return -1;
  // measured at the Large, one-GPU-share and Mid shapes: the register-staged 256 x 256 tile (0) is the fastest for
  // every epilogue; the direct-to-LDS variants (10, 11) stay reachable through the tuning override
  static const int big[] = {0, 4, 2, -1}, big_qkv[] = {0, 10, 8, 4, 2, -1}, mid[] = {4, 2, -1}, m64[] = {3, 6, -1}, m32[] = {5, 7, -1};
  const int* cand;
  // grouped GEMM: the tile height follows the rows of an average group, not the padded total
  const int m_sel = g.blk_group && g.grp_rows > 0 && g.grp_rows < g.M ? g.grp_rows : g.M;
  if (m_sel <= 32) cand = m32;
  else if (m_sel <= 64) cand = m64;
  else if (m_sel <= 128 || (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256) * g.batch < 200) cand = mid;
  else cand = g.epi == EPI_QKV ? big_qkv : big;
  if (pt_tune_gemm_cfg >= 0 && pt_tune_gemm_cfg < GM_NCFG) return cfg_fits(g, pt_tune_gemm_cfg) ? pt_tune_gemm_cfg : -1;
  for (; *cand >= 0; ++cand)
    if (cfg_fits(g, *cand)) return *cand;
  return -1;
}

bool pt_gemm_mfma_covers(const pt_gemm_args& g) { return choose_cfg(g) >= 0; }

// Configurations whose tile is at least 128 x 128 run the LDS-staged residual epilogue, which can also emit the
// scaled bf16 copy and the per-row sums of squares; one block of sums per wavefront column range.
int pt_gemm_mfma_fold_parts(const pt_gemm_args& g) {
  if (g.epi != EPI_RESIDUAL) return 0;
  const int cfg = choose_cfg(g);
  static const bool staged[GM_NCFG] = {true, true, true, false, true, false, false, false, true, true, true, true};
  if (cfg < 0 || !staged[cfg] || g.N % kWaveN[cfg]) return 0;
  return g.N / kWaveN[cfg];
}

int pt_launch_gemm_mfma(const pt_gemm_args& g, hipStream_t s) {
  const int cfg = choose_cfg(g);
  if (cfg == -2) return 1;
  if (cfg < 0) return 0;
  if (g.nf_out && g.nf_parts != pt_gemm_mfma_fold_parts(g))
    return pt_set_error(PT_ERR_INVALID_ARGUMENT, "folded RMSNorm asked of a GEMM configuration that cannot emit it");
  switch (g.epi) {
    case EPI_STORE_F32: return launch_epi<EPI_STORE_F32>(g, s, cfg);
    case EPI_RESIDUAL: return launch_epi<EPI_RESIDUAL>(g, s, cfg);
    case EPI_SWIGLU: return launch_epi<EPI_SWIGLU>(g, s, cfg);
    case EPI_QKV: return launch_epi<EPI_QKV>(g, s, cfg);
  }
  return 0;
}

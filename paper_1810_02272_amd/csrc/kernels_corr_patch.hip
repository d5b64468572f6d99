// Patch-staged implicit-GEMM correlation kernel for gfx950: a variant of corr_kernel for
// stride-1, dilation-1 gathers whose channel count per group is a multiple of 8 (forward of such
// layers, and every backward-data pass, which is always a stride-1 correlation over dy).  It is
// selected where the gather kernel spends the most per gathered element -- the 256-column tiles of
// at most 48 rows (e.g. the 48-row backward-data GEMM of a grouped 5x5 layer) -- and, for kernels of
// 25 taps or more (every patch element is then used 25 times), on the 128x128 and 32x128 tiles;
// elsewhere the gather kernel measured equal or faster.
//
//   D[m][col] = sum_k A[m][k] * in[n, g*Cg + c, a - ph + i, b - pw + j],  k = (c, i, j), col = (n, a, b)
//
// Instead of gathering every (k, col) element from memory (each input element kh*kw times), a
// workgroup keeps the raw input rows its columns touch -- a zero-padded "patch" of 8 channels at a
// time -- in LDS, and the MFMA B operand is read straight out of the patch: the element of column
// (a, b) under tap (i, j) sits at patch[(a + i) * PWID + b + j], so a lane's address is its
// column's base plus a tap offset that is uniform over the wave.  Padding, ragged image borders
// and columns past the batch are resolved once, when the patch is loaded (hardware range-checked
// buffer loads return the zeros); the inner loop has no bounds logic and almost no vector-memory
// traffic.  The reduction runs in the order (8-channel chunk, tap, channel in chunk): one "super
// step" is one tap of 8 channels, and the weights are packed in the same order.
#include <hip/hip_runtime.h>

#include "corr_epilogue.h"
#include "device_utils.h"
#include "internal.h"

namespace mi355conv {

namespace {

constexpr int kThreads = 256;

template <int MT, int MB, int NB, int WM, int WN>
struct PatchCfg {
  static constexpr int BK = 16;  // k per A chunk: two super steps
  static constexpr int LDK = BK + 4;
  static constexpr int BM = WM * MB * MT;
  static constexpr int BN = WN * NB * MT;
  static constexpr int LG = 64 / MT;  // lane groups along k of one MFMA
  static constexpr int CPG = 8 / LG;  // channels of a super step each lane group multiplies (4 or 2)
  static constexpr int A_WI = BM / 16;
  static constexpr int A_PER = (A_WI + 3) / 4;
  static constexpr int ASTAGE = BM * LDK;
  static constexpr int NKS = 2 * CPG;  // MFMA k steps per A chunk
  static_assert(WM * WN == 4, "four waves per workgroup");
};

template <int MT, int MB, int NB, int WM, int WN>
__global__ __launch_bounds__(kThreads) void corr_patch_kernel(const CorrArgs a) {
  using C = PatchCfg<MT, MB, NB, WM, WN>;
  using M = Mfma<MT>;
  constexpr int BM = C::BM, BN = C::BN, LDK = C::LDK, CPG = C::CPG, NKS = C::NKS;
  constexpr int EPT = kPatchEPT;
  typedef float vec_a __attribute__((ext_vector_type(CPG)));

  extern __shared__ __align__(16) float smem[];  // [2][BM][LDK] A stages, then [2][8][PSZ] patch stages
  const uint32_t patch_bytes0 = 2u * C::ASTAGE * 4u;

  const int t = threadIdx.x;
  const int lane = t & 63;
  const int wv = __builtin_amdgcn_readfirstlane(t >> 6);
  const int wm = wv / WN, wn = wv % WN;

  uint32_t lin = xcd_contiguous_block_id();
  const uint32_t m_tile = lin % (uint32_t)a.m_tiles;
  lin /= (uint32_t)a.m_tiles;
  const uint32_t col_tile = lin % (uint32_t)a.col_tiles;
  const uint32_t g = lin / (uint32_t)a.col_tiles;

  // ---- geometry of this tile's patch (uniform) ---------------------------------------------
  // The tile's columns run through one or more images ("segments").  Segment 0 starts at output
  // row a0 of image n0 and owns patch rows 0 .. R0-1; every later segment starts at output row 0
  // and owns RS = PH + TH - 1 patch rows.  Patch row r of a segment that starts at output row alo
  // is input row alo - ph + r; patch column c is input column c - pw.
  const int TH = a.THW / a.TW;
  const uint32_t col0 = col_tile * BN;
  const uint32_t n0 = mdiv(col0, a.mP);
  const uint32_t a0 = mdiv(col0 - n0 * a.P, a.mPW);
  const uint32_t R0 = (uint32_t)a.PH - a0 + TH - 1;
  const uint32_t RS = (uint32_t)a.PH + TH - 1;
  auto patch_row_base = [&](uint32_t n, uint32_t pa) {  // patch row of output row pa of image n
    const uint32_t s = n - n0;
    return s == 0 ? pa - a0 : R0 + (s - 1) * RS + pa;
  };
  uint32_t col_last = col0 + BN - 1;
  if (col_last > (uint32_t)a.ncols - 1) col_last = (uint32_t)a.ncols - 1;
  uint32_t patch_elems;  // floats of one channel of this tile's patch
  {
    const uint32_t n = mdiv(col_last, a.mP);
    const uint32_t pa = mdiv(col_last - n * a.P, a.mPW);
    patch_elems = (patch_row_base(n, pa) + TH) * (uint32_t)a.PWID;
  }

  // ---- per-lane B columns: byte address of (column, channels CPG*h .. CPG*h + CPG-1) inside a patch
  // stage.  A stage is [lane group h][position][CPG channels]: the CPG channels one lane multiplies at a
  // super step sit side by side, so its B operands are one 8- or 16-byte read, and 16 (or 32)
  // consecutive columns of a lane group are one contiguous run of LDS.
  uint32_t lanebase[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    uint32_t col = col0 + (wn * NB + j) * MT + lane % MT;
    if (col > col_last) col = col_last;  // columns past the edge are never stored: any valid address
    const uint32_t n = mdiv(col, a.mP);
    const uint32_t pix = col - n * a.P;
    const uint32_t pa = mdiv(pix, a.mPW);
    const uint32_t pb = pix - pa * a.PW;
    const uint32_t cb = patch_row_base(n, pa) * (uint32_t)a.PWID + pb;
    lanebase[j] = patch_bytes0 + 4u * (uint32_t)CPG * (cb + (uint32_t)(lane / MT) * (uint32_t)a.PSZ);
  }

  // ---- per-thread patch elements: where they come from (relative to channel 0 of the group) --
  const __amdgpu_buffer_rsrc_t in_rsrc =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(a.in), 0, (int)a.in_bytes, 0x00020000);
  uint32_t psrc[EPT];
#pragma unroll
  for (int r = 0; r < EPT; ++r) {
    const uint32_t e = t + r * kThreads;
    uint32_t src = 0x80000000u;  // beyond the blob (which is at most 2^30 bytes): reads as zero
    if (e < patch_elems) {
      const uint32_t prow = mdiv(e, a.mPWID);
      const uint32_t pcol = e - prow * a.PWID;
      uint32_t n = n0, rin = prow, alo = a0;
      if (prow >= R0) {
        const uint32_t s1 = mdiv(prow - R0, a.mRSEG);
        n = n0 + 1 + s1;
        rin = prow - R0 - s1 * RS;
        alo = 0;
      }
      const int ih = (int)(alo + rin) - a.ph, iw = (int)pcol - a.pw;
      if ((uint32_t)ih < (uint32_t)a.IH && (uint32_t)iw < (uint32_t)a.IW && n < (uint32_t)a.Nimg)
        src = 4u * (n * (uint32_t)a.in_img_stride + g * (uint32_t)a.in_grp_stride + (uint32_t)ih * a.IW + iw);
    }
    psrc[r] = src;
  }
  const uint32_t chan_bytes = 4u * (uint32_t)a.IHW;
  float pr[8][EPT];
  auto patch_load = [&](int cc) {
    const uint32_t coff = (uint32_t)(cc * 8) * chan_bytes;
#pragma unroll
    for (int c8 = 0; c8 < 8; ++c8)
#pragma unroll
      for (int r = 0; r < EPT; ++r)
        pr[c8][r] = __builtin_bit_cast(
            float, __builtin_amdgcn_raw_buffer_load_b32(in_rsrc, psrc[r] + coff + c8 * chan_bytes, 0, 0));
  };
  auto patch_store = [&](int buf) {
    float* dst = smem + 2 * C::ASTAGE + buf * 8 * a.PSZ;
#pragma unroll
    for (int h = 0; h < C::LG; ++h)
#pragma unroll
      for (int r = 0; r < EPT; ++r)
        if (t + r * kThreads < (uint32_t)a.PSZ) {
          vec_a v;
#pragma unroll
          for (int u = 0; u < CPG; ++u) v[u] = pr[CPG * h + u][r];
          *reinterpret_cast<vec_a*>(dst + (h * a.PSZ + t + r * kThreads) * CPG) = v;
        }
  };

  // ---- A tile staging: as in corr_kernel ([row][k], 16 bytes per lane, four chunks deep) -----
  const float* Ag = a.A + ((size_t)g * a.MP + (size_t)m_tile * BM) * a.KP;
  const int arow = (lane & 7) + 8 * (lane >> 5), ac4 = (lane >> 3) & 3;
  uint32_t aoff[C::A_PER];
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) aoff[p] = 4u * (uint32_t)(((wv + 4 * p) * 16 + arow) * a.KP + ac4 * 4);
  f32x4 raX[C::A_PER], raY[C::A_PER];
  auto load_a = [&](f32x4(&ra)[C::A_PER], int kc, int p) {
    if (C::A_WI % 4 == 0 || wv + 4 * p < C::A_WI)
      ra[p] = *reinterpret_cast<const f32x4*>(reinterpret_cast<const char*>(Ag) + (aoff[p] + (uint32_t)kc * 64u));
  };
  auto store_a = [&](f32x4(&ra)[C::A_PER], int buf, int p) {
    if (C::A_WI % 4 == 0 || wv + 4 * p < C::A_WI)
      *reinterpret_cast<f32x4*>(smem + buf * C::ASTAGE + ((wv + 4 * p) * 16 + arow) * LDK + ac4 * 4) = ra[p];
  };

  typename M::Acc acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < M::NR; ++r) acc[i][j][r] = 0.f;

  // ---- prologue ----------------------------------------------------------------------------
  const int nchunks = a.KP / C::BK;
  const int last = nchunks - 1;
  patch_load(0);
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) load_a(raX, 0, p);
  patch_store(0);
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) store_a(raX, 0, p);
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) load_a(raX, last < 1 ? last : 1, p);
#pragma unroll
  for (int p = 0; p < C::A_PER; ++p) load_a(raY, last < 2 ? last : 2, p);
  __syncthreads();

  // ---- main loop: one iteration = one A chunk = two super steps -------------------------------
  // Reduction state (uniform): channel chunk cc, tap index tap = ti*TW + tj inside it.
  int cc = 0, tap = 0, ti = 0, tj = 0, sg = 0;
  const int T = a.THW, tstore = a.THW / 2;
  const float* opA = smem + (wm * MB * MT + lane % MT) * LDK + (lane / MT) * CPG;
  const uint32_t stage_bytes = 4u * 8u * (uint32_t)a.PSZ;

  auto iteration = [&](int kc, f32x4(&ra)[C::A_PER]) {
    const int cur = kc & 1, nxt = cur ^ 1;
    const int kld = kc + 3 < last ? kc + 3 : last;
    const float* sA = opA + cur * C::ASTAGE;
    vec_a av[2][MB];
#pragma unroll
    for (int ssl = 0; ssl < 2; ++ssl)
#pragma unroll
      for (int i = 0; i < MB; ++i) av[ssl][i] = *reinterpret_cast<const vec_a*>(sA + i * MT * LDK + ssl * 8);
#pragma unroll
    for (int ssl = 0; ssl < 2; ++ssl) {
      if (sg < a.NS) {  // the last chunk of an odd number of super steps has only one
        const uint32_t soff = (uint32_t)(cc & 1) * stage_bytes + 4u * (uint32_t)CPG * (uint32_t)(ti * a.PWID + tj);
        vec_a bv[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j)
          bv[j] = *reinterpret_cast<const vec_a*>(reinterpret_cast<const char*>(smem) + (lanebase[j] + soff));
#pragma unroll
        for (int u = 0; u < CPG; ++u) {
#pragma unroll
          for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < NB; ++j) M::run(av[ssl][i][u], bv[j][u], acc[i][j]);
          // this step's share of the A staging work
#pragma unroll
          for (int p = 0; p < C::A_PER; ++p)
            if ((p * NKS + NKS / 2) / C::A_PER % NKS == ssl * CPG + u) {
              store_a(ra, nxt, p);
              load_a(ra, kld, p);
            }
          __builtin_amdgcn_sched_barrier(0);
        }
        // Patch of the next channel chunk: requested at the first tap of this one and written to the
        // other patch stage half way through -- with at least 3 taps that is at least one barrier
        // after that stage's last reader and at least one before its first.
        if (tap == 0 && (cc + 1) * 8 < a.Cg_in) patch_load(cc + 1);
        if (tap == tstore && (cc + 1) * 8 < a.Cg_in) patch_store((cc + 1) & 1);
        ++sg;
        ++tap;
        if (++tj == a.TW) {
          tj = 0;
          ++ti;
        }
        if (tap == T) {
          tap = 0;
          ti = 0;
          ++cc;
        }
      }
    }
    __syncthreads();
  };

  int kc = 0;
  for (; kc + 1 < nchunks; kc += 2) {
    iteration(kc, raX);
    iteration(kc + 1, raY);
  }
  if (kc < nchunks) iteration(kc, raX);

  corr_epilogue<MT, MB, NB, BM, BN>(a, smem, acc, m_tile, col_tile, g, wm, wn);
}

template <int MT, int MB, int NB, int WM, int WN>
int launch_patch_t(const CorrArgs& a, hipStream_t s) {
  using C = PatchCfg<MT, MB, NB, WM, WN>;
  const size_t lds = (size_t)(2 * C::ASTAGE + 16 * a.PSZ) * 4;
  static LdsOptIn opt_in;  // more than 64 KB of LDS needs an explicit opt-in, once per process
  if (const int e = lds_opt_in(opt_in, &corr_patch_kernel<MT, MB, NB, WM, WN>, 160 * 1024)) return e;
  const uint32_t blocks = (uint32_t)a.G * a.m_tiles * a.col_tiles;
  hipLaunchKernelGGL((corr_patch_kernel<MT, MB, NB, WM, WN>), dim3(blocks), dim3(kThreads), lds, s, a);
  return (int)hipGetLastError();
}

}  // namespace

int launch_corr_patch(int32_t tile, const CorrArgs& a, void* stream) {
  hipStream_t s = (hipStream_t)stream;
  switch (tile) {  // the tiles configure_patch (api.cpp) may select
    //                                       MT MB NB WM WN
    case CORR_128x128: return launch_patch_t<32, 2, 2, 2, 2>(a, s);
    case CORR_32x128:  return launch_patch_t<32, 1, 1, 1, 4>(a, s);
    case CORR_32x256:  return launch_patch_t<32, 1, 2, 1, 4>(a, s);
    case CORR_48x256:  return launch_patch_t<16, 3, 4, 1, 4>(a, s);
    case CORR_16x256:  return launch_patch_t<16, 1, 4, 1, 4>(a, s);
    default: return (int)hipErrorInvalidValue;
  }
}

}  // namespace mi355conv
